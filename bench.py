#!/usr/bin/env python3
"""Throughput of the RDK redistribute + verify path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic inputs that already sit in HBM:
redistribution with the top-k sparse kernel (Alg. 1 steps 1-2) and verification (Alg. 4), through the fused
entry point rdk_redistribute_verify (default) or as rdk_redistribute_linear -> rdk_verify_sample.
Prints ONE JSON line: positions/s, the roofline of the dominant kernel (timed live with HIP events
inside the library), and the CPU oracle timed on a bounded sample of the same workload.  Unless --no-extra is
given, "extra" also carries the other linear form (Eq. 3) on the same batch and the exact dense products (bf16 at
N=256000, n=32000, B=512; fp32 at N=32000, n=8000, B=64) against the MFMA peaks.

  python bench.py [--steps K] [--warmup W] [--mode sparse|taylor] [--path fused|twocall] [--workload NAME] [--no-cpu] [--no-extra]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
MFMA_F32_PEAK_TFLOPS = 157.3    # MI355X fp32 matrix, published


# HBM bytes per launch from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this script (summary and
# commands in profiles/), scaled by the 256 MiB yardstick pass below: bytes = 1024 * (2 * FETCH_SIZE + WRITE_SIZE).
# Keyed by (workload, mode, path, kernel); valid for the kernels as committed with that summary.
MEASURED_TRAFFIC = {
    ("llama3", "sparse", "fused", "sparse_product_kernel"): 490.7e6,
    ("llama3", "taylor", "fused", "taylor_stats_kernel"): 167.2e6,
    ("llama3", "taylor", "fused", "taylor_write_kernel"): 166.8e6,
    ("dense256k", "exact", "bf16", "exact_bf16_kernel"): 19206.4e6,
    ("n32k", "exact", "f32", "exact_f32_split_kernel"): 1085.3e6,
    ("llama3", "multi", "C4", "verify_multi_kernel"): 483.5e6,
}


def algorithmic_bytes(kernel, w, B, kk, fused, esz):
    """Bytes one launch of a kernel must move for B positions (inputs read once, outputs written once).
    esz = bytes per input element (4: fp32, 2: bf16 logits).  In the fused path the product / Eq. 3 kernels
    read p instead of writing q'."""
    N, n = w.N, w.n
    tables = 8 * (N - n) * kk + 4 * n + 4 * N                               # neighbour rows, diagonal, id maps: once
    ids = 4 * n + 4 * ((N + 1023) // 1024 + 1)                              # kept ids and first slot per chunk: once
    return {
        "verify_stream_kernel": B * (esz + 4) * N,                          # read p and q'
        "sparse_product_kernel": B * ((esz if fused else 4) * N + 4 * n) + tables,   # read q^T, p (fused) or write q'
        "taylor_stats_kernel": B * esz * (N + n) + ids,                     # read p, q
        "taylor_write_kernel": B * (esz * (N + n) + (0 if fused else 4 * N)) + ids,
        "taylor_row_kernel": B * esz * (N + n) + ids,                       # one pass: p and q read once
        "q_transpose_kernel": B * (esz + 4) * n,
        "row_stats_kernel": B * esz * n,
        "verify_finalize_kernel": B * 3 * 4 * ((N + 1023) // 1024),
    }.get(kernel)


def run_linear(args, rdk, synth, torch, w, vocab, batch, mode_name, path, steps, warmup):
    """Times `steps` passes of redistribution (mode_name) + verification over the batch; returns the figures."""
    bias, kept, E = vocab
    B = w.B
    dev = torch.device("cuda:0")
    kept_d = torch.from_numpy(kept).to(dev)
    t0 = time.time()
    if mode_name == "sparse":
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
    outs = [torch.empty((B, w.N), dtype=torch.float32, device=dev) for _ in range(C)] if path == "twocall" else None
    vout = rdk.VerifyOutputs(B, w.N, w.gamma, dev)
    kern.workspace(B)
    mode = rdk.LINEAR_SPARSE if mode_name == "sparse" else rdk.LINEAR_TAYLOR
    fused = path == "fused"

    def step(i):
        c = i % C
        if fused:
            rdk.rdk_redistribute_verify(kern, mode, ps[c], qs[c], seed=2506, offset=i * B, gamma=w.gamma, p_kind=kind,
                                        q_kind=kind, outputs=vout)
        else:
            rdk.rdk_redistribute_linear(kern, mode, qs[c], kind, p=ps[c] if mode_name == "taylor" else None, p_kind=kind,
                                        out=outs[c])
            rdk.rdk_verify_sample(ps[c], outs[c], seed=2506, offset=i * B, gamma=w.gamma, p_kind=kind, outputs=vout)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    # which kernel dominates?  a short pass with every kernel bracketed by events
    names = ["row_stats_kernel", "q_transpose_kernel", "sparse_product_kernel", "taylor_stats_kernel", "taylor_write_kernel",
             "taylor_row_kernel", "verify_stream_kernel", "verify_finalize_kernel"]
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
    for i in range(steps):
        step(warmup + i)
    stop.record()
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    total_ms = start.elapsed_time(stop)
    cnt, kms = rdk.rdk_timing_read(dominant)
    ms_per_step = total_ms / steps

    kk = (max(w.k, 1) + 15) // 16 * 16
    esz = 2 if w.logits_bf16 else 4
    alg = algorithmic_bytes(dominant, w, B, kk, fused, esz)
    avg_s = kms / cnt * 1e-3
    achieved = alg / avg_s / 1e9
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get((w.name, mode_name, path, dominant)),
                "avg_launch_us": round(avg_s * 1e6, 2),
                "algorithmic_bytes_per_launch": alg}
    # whole-step compulsory bytes: fused = read p and q once; two calls = q read, q' written then read, p read (twice for Eq. 3)
    if fused:
        step_bytes = B * esz * (w.N + w.n) + (8 * (w.N - w.n) * kk if mode_name == "sparse" else 0)
    else:
        step_bytes = B * (esz * (w.n + w.N) + 8 * w.N) + (8 * (w.N - w.n) * kk if mode_name == "sparse" else B * esz * w.N)
    res_extra = {}
    if dominant == "sparse_product_kernel":
        # what the kernel is limited by: 128-byte lines gathered from q^T through the vector L1 (one per neighbour and
        # 32 positions), against 64 bytes per clock and compute unit (256 units, 2.4 GHz)
        lines = (w.N - w.n) * kk * ((B + 31) // 32)
        l1_peak = 256 * 64 * 2.4          # GB/s
        measured = 246.0e9 * 128 / 1e9    # GB/s: the bare line-gather loop of the `ceilings` program (profiles/ceilings_mi355x.md)
        res_extra["sparse_gather"] = {"lines_per_launch": lines, "achieved_GBs": round(lines * 128 / avg_s / 1e9, 1),
                                      "vector_l1_peak_GBs": round(l1_peak, 1),
                                      "frac": round(lines * 128 / avg_s / 1e9 / l1_peak, 4),
                                      "bare_gather_loop_GBs": round(measured, 1),
                                      "frac_of_bare_gather_loop": round(lines * 128 / avg_s / 1e9 / measured, 4)}
    return {"ms_per_step": ms_per_step, "value": B / (ms_per_step * 1e-3), "roofline": roofline, **res_extra,
            "kernels": {k: {"avg_us": round(v["avg_us"], 2), "per_step": v["launches_per_step"]} for k, v in per_kernel.items()},
            "step_algorithmic_GBs": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
            "step_frac_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "kernel_build_s": round(build_s, 3),
            "accept_rate": float(vout.accept.float().mean().item()), "mean_alpha": float(vout.alpha.mean().item())}


def run_draft(args, rdk, synth, torch, w, vocab, batch, steps):
    """Draft-side sampling alone: rdk_sample_draft with the top-k sparse kernel, q' never materialised."""
    bias, kept, E = vocab
    dev = torch.device("cuda:0")
    kern = rdk.rdk_build_kernel(w.N, torch.from_numpy(kept).to(dev), rdk.SPARSE_TOPK, embeddings=torch.from_numpy(E).to(dev),
                                tau=w.tau, k=w.k)
    if w.logits_bf16:
        q_host, kind = torch.from_numpy(batch["z_q"]).to(torch.bfloat16), "logit"
    else:
        q_host, kind = torch.from_numpy(batch["q_hat"]), "prob"
    qs = [q_host.to(dev) for _ in range(max(1, args.copies))]
    ids = torch.empty(w.B, dtype=torch.int32, device=dev)
    qd = torch.empty(w.B, dtype=torch.float32, device=dev)
    for i in range(5):
        rdk.rdk_sample_draft(kern, qs[i % len(qs)], 2506, i * w.B, kind, draft_ids=ids, q_draft=qd)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(steps):
        rdk.rdk_sample_draft(kern, qs[i % len(qs)], 2506, i * w.B, kind, draft_ids=ids, q_draft=qd)
    stop.record()
    torch.cuda.synchronize()
    ms = start.elapsed_time(stop) / steps
    return {"entry": "rdk_sample_draft (sparse top-k, no target row)", "ms_per_step": round(ms, 5),
            "positions_per_s": round(w.B / (ms * 1e-3), 1)}


def run_multi(args, rdk, synth, torch, w, vocab, batch, steps, C=4):
    """Several candidates per position (rdk_verify_multi) on the materialised rows of the sparse form: the candidates
    drawn from q', then one pass over p and q' per rejected candidate."""
    bias, kept, E = vocab
    dev = torch.device("cuda:0")
    kern = rdk.rdk_build_kernel(w.N, torch.from_numpy(kept).to(dev), rdk.SPARSE_TOPK, embeddings=torch.from_numpy(E).to(dev),
                                tau=w.tau, k=w.k)
    if w.logits_bf16:
        p_host, q_host, kind = torch.from_numpy(batch["z_p"]).to(torch.bfloat16), torch.from_numpy(batch["z_q"]).to(torch.bfloat16), "logit"
    else:
        p_host, q_host, kind = torch.from_numpy(batch["p"]), torch.from_numpy(batch["q_hat"]), "prob"
    n_copies = max(1, args.copies)
    ps = [p_host.to(dev) for _ in range(n_copies)]
    qp = [rdk.rdk_redistribute_linear(kern, rdk.LINEAR_SPARSE, q_host.to(dev), kind) for _ in range(n_copies)]
    out = rdk.MultiOutputs(w.B, C, dev)
    for i in range(5):
        rdk.rdk_verify_multi(ps[i % n_copies], qp[i % n_copies], C, 2506, i * w.B, kind, outputs=out)
    torch.cuda.synchronize()
    rdk.rdk_timing_select("verify_multi_kernel")
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(steps):
        rdk.rdk_verify_multi(ps[i % n_copies], qp[i % n_copies], C, 2506, i * w.B, kind, outputs=out)
    stop.record()
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    ms = start.elapsed_time(stop) / steps
    cnt, kms = rdk.rdk_timing_read("verify_multi_kernel")
    # passes of the last step: one over q' for the candidates, one over p and q' per rejection
    rejections = float(torch.minimum(out.accepted, torch.full_like(out.accepted, C)).float().mean().item())
    esz = 2 if w.logits_bf16 else 4
    alg = w.B * (4.0 * w.N + rejections * (4.0 + esz) * w.N)
    gbs = alg / (kms / cnt * 1e-3) / 1e9
    return {"entry": "rdk_verify_multi, C=%d candidates per position, q' materialised" % C, "ms_per_step": round(ms, 5),
            "positions_per_s": round(w.B / (ms * 1e-3), 1), "mean_rejections_per_position": round(rejections, 3),
            "kept_one_of_C": round(float((out.accepted < C).float().mean().item()), 4),
            "roofline": {"kernel": "verify_multi_kernel", "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                         "traffic": MEASURED_TRAFFIC.get((w.name, "multi", "C%d" % C, "verify_multi_kernel")),
                         "avg_launch_us": round(kms / cnt * 1e3, 2), "algorithmic_bytes_per_launch": alg}}


def run_exact(rdk, synth, torch, wname, fmt, calls=5):
    """Exact dense redistribution (Alg. 1 with the full M): bf16 MFMA contraction at N=256000, n=32000, B=512 (bound by
    the matrix cores), or the fp32 one at N=32000, n=8000, B=64 (three bf16 parts per operand on the bf16 matrix cores:
    bound by streaming M from HBM once)."""
    w = synth.WORKLOADS[wname]
    dev = torch.device("cuda:0")
    bias, kept, E, rng = synth.make_vocab(w)
    batch = synth.make_batch(w, bias, kept, rng)
    kern = rdk.rdk_build_kernel(w.N, torch.from_numpy(kept).to(dev), rdk.DENSE_BF16 if fmt == "bf16" else rdk.DENSE_F32,
                                embeddings=torch.from_numpy(E).to(dev), tau=w.tau)
    q = torch.from_numpy(batch["q_hat"]).to(dev)
    out = torch.empty((w.B, w.N), dtype=torch.float32, device=dev)
    for _ in range(2):
        rdk.rdk_redistribute_exact(kern, q, out=out)
    torch.cuda.synchronize()
    kname = "exact_bf16_kernel" if fmt == "bf16" else "exact_f32_split_kernel"
    rdk.rdk_timing_select(kname)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(calls):
        rdk.rdk_redistribute_exact(kern, q, out=out)
    stop.record()
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    ms_call = start.elapsed_time(stop) / calls
    cnt, kms = rdk.rdk_timing_read(kname)
    flops = 2.0 * w.B * w.n * w.N
    k_tf = flops / (kms / cnt * 1e-3) / 1e12
    row_err = float((out.double().sum(1) - 1).abs().max().item())
    esz = 2 if fmt == "bf16" else 4
    del kern, out, q
    torch.cuda.empty_cache()
    traffic = MEASURED_TRAFFIC.get((wname, "exact", fmt, kname))
    if fmt == "bf16":
        roofline = {"kernel": kname, "bound": "mfma", "achieved": round(k_tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(k_tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                    "avg_launch_us": round(kms / cnt * 1e3, 1), "algorithmic_flops_per_launch": flops}
    else:
        # M read once, the drafter rows read once, the output written once (the split partials are not counted)
        alg = 4.0 * w.n * w.N + 4.0 * w.B * (w.n + w.N)
        gbs = alg / (kms / cnt * 1e-3) / 1e9
        roofline = {"kernel": kname, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "avg_launch_us": round(kms / cnt * 1e3, 1),
                    "algorithmic_bytes_per_launch": alg, "algorithmic_TFLOPs": round(k_tf, 1),
                    "fp32_matrix_peak_TFLOPs": MFMA_F32_PEAK_TFLOPS}
    return {"workload": "%s: N=%d n=%d B=%d, M %s %.2f GB" % (wname, w.N, w.n, w.B, fmt, esz * w.n * w.N / 1e9),
            "ms_per_call": round(ms_call, 3), "positions_per_s": round(w.B / (ms_call * 1e-3), 1), "roofline": roofline,
            "call_TFLOPs": round(flops / (ms_call * 1e-3) / 1e12, 1), "max_row_sum_error": row_err}


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
    ap.add_argument("--no-extra", action="store_true", help="skip the other linear form and the exact bf16 product")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this library runs on one GPU (positions are independent: shard the batch); run with --gpus 1")

    import torch
    from paper_2506_03206_amd import rdk, synth

    wname = args.workload or "llama3"
    w = synth.WORKLOADS[wname]
    B = w.B
    torch.cuda.set_device(0)

    # Yardstick for hardware byte counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE): one elementwise pass that
    # reads exactly 256 MiB and writes exactly 256 MiB; it is the only launch with 2^26 float elements.
    cal = torch.zeros(1 << 26, dtype=torch.float32, device="cuda:0")
    cal_out = torch.empty_like(cal)
    torch.add(cal, 1.0, out=cal_out)
    torch.cuda.synchronize()
    del cal, cal_out
    torch.cuda.empty_cache()

    t0 = time.time()
    bias, kept, E, rng = synth.make_vocab(w)
    batch = synth.make_batch(w, bias, kept, rng)
    gen_s = time.time() - t0

    r = run_linear(args, rdk, synth, torch, w, (bias, kept, E), batch, args.mode, args.path, args.steps, args.warmup)
    extra = {k: r[k] for k in ("kernels", "step_algorithmic_GBs", "step_frac_of_hbm_peak", "kernel_build_s", "accept_rate",
                               "mean_alpha")}
    extra["input_gen_s"] = round(gen_s, 2)
    if "sparse_gather" in r:
        extra["sparse_gather"] = r["sparse_gather"]
    if not args.no_extra:
        other = "taylor" if args.mode == "sparse" else "sparse"
        torch.cuda.empty_cache()
        o = run_linear(args, rdk, synth, torch, w, (bias, kept, E), batch, other, args.path, max(20, args.steps // 2), args.warmup)
        extra["other_linear_form"] = {"mode": other, "path": args.path, "positions_per_s": round(o["value"], 1),
                                      "ms_per_step": round(o["ms_per_step"], 5), "roofline": o["roofline"], "kernels": o["kernels"],
                                      "step_frac_of_hbm_peak": o["step_frac_of_hbm_peak"]}
        if "sparse_gather" in o:
            extra["other_linear_form"]["sparse_gather"] = o["sparse_gather"]
        extra["draft_sampling"] = run_draft(args, rdk, synth, torch, w, (bias, kept, E), batch, max(20, args.steps // 2))
        extra["multi_candidate"] = run_multi(args, rdk, synth, torch, w, (bias, kept, E), batch, max(20, args.steps // 4))
        torch.cuda.empty_cache()
        extra["exact_bf16"] = run_exact(rdk, synth, torch, "dense256k", "bf16", calls=10)
        extra["exact_f32"] = run_exact(rdk, synth, torch, "n32k", "f32", calls=20)

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(args, w, batch, kept)

    line = {"metric": "redistribute+verify positions/sec at N=%d, n=%d" % (w.N, w.n), "value": round(r["value"], 1),
            "unit": "positions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(r["ms_per_step"], 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": "%s: N=%d n=%d B=%d (%d seqs x %d drafts) k=%d, %s linear RDK + verify/sample, %s inputs"
                       % (w.name, w.N, w.n, B, w.seqs, w.gamma, w.k, args.mode, "bf16 logit" if w.logits_bf16 else "fp32 prob"),
                       "mode": args.mode, "path": args.path, "N": w.N, "n": w.n, "B": B, "k": w.k},
            "roofline": r["roofline"], "cpu_baseline": cpu, "extra": extra}
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
