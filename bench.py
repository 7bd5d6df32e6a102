#!/usr/bin/env python3
"""Throughput of the RDK redistribute + verify path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic inputs that already sit in HBM:
redistribution with the top-k sparse kernel (Alg. 1 steps 1-2) and verification (Alg. 4), through the fused
entry point rdk_redistribute_verify (default) or as rdk_redistribute_linear -> rdk_verify_sample.
The timed region of K steps is run five times; the line reports the median region.  Prints ONE JSON line:
positions/s, the roofline of the dominant kernel (timed live with HIP events inside the library), and the CPU oracle
timed on a bounded sample of the same workload (one thread, and one worker process per host core).  Unless --no-extra
is given, "extra" also carries the other linear form (Eq. 3) on the same batch, the draft draw, several candidates per
position, the small exact workload (N=32000: exact fp32 product and both fused linear forms), the extreme-pruning
workload (N=151936, bf16 logits, both fused forms) and the dense workload (N=256000: exact 16-bit product against
the matrix-core peak, and both fused linear forms on the same inputs).

  python bench.py [--steps K] [--warmup W] [--mode sparse|taylor] [--path fused|twocall] [--workload NAME] [--no-cpu] [--no-extra]
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 / fp16 matrix rate, published
MFMA_F32_PEAK_TFLOPS = 157.3    # MI355X fp32 matrix, published
REPEATS = 5                     # timed regions per measurement; the median is reported
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def kernel_source_hash():
    """Hash of the kernel sources: the counter figures in profiles/hbm_traffic.json are valid for one state of them."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2506_03206_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".hpp")) and name != "ceilings.hip":
            with open(os.path.join(csrc, name), "rb") as fh:
                h.update(name.encode())
                h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic():
    """HBM bytes per launch from the rocprofv3 counter runs recorded in profiles/hbm_traffic.json (kernel -> bytes), or an
    empty table when the kernel sources have changed since the counters were taken."""
    try:
        with open(TRAFFIC_FILE) as fh:
            rec = json.load(fh)
    except (OSError, ValueError):
        return {}, None
    if rec.get("kernel_source_hash") != kernel_source_hash():
        return {}, "stale: kernel sources changed since profiles/hbm_traffic.json was taken"
    return {tuple(k.split("|")): v for k, v in rec.get("bytes_per_launch", {}).items()}, rec.get("taken_at_commit")


def softmax_rows(z):
    """Input preparation on the benchmark's side: probability rows from logit rows (fp64, then fp32)."""
    z = z.astype(np.float64)
    z -= z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def prob_inputs(batch, kept):
    """Target probabilities p [B,N] and the drafter's full-vocabulary probabilities on the kept ids q_hat [B,n] (rows
    sum to less than one: Eq. 1 has work to do)."""
    if "p" not in batch:
        batch["p"] = softmax_rows(batch["z_p"]).astype(np.float32)
        batch["q_hat"] = np.ascontiguousarray(softmax_rows(batch["z_d"])[:, kept], dtype=np.float32)
    return batch["p"], batch["q_hat"]


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
        "sequence_scan_kernel": B * 9,
    }.get(kernel)


KERNEL_NAMES = ["row_stats_kernel", "q_transpose_kernel", "sparse_product_kernel", "taylor_stats_kernel", "taylor_write_kernel",
                "taylor_row_kernel", "verify_stream_kernel", "verify_finalize_kernel", "sequence_scan_kernel"]


def timed_regions(torch, fn, steps, first):
    """REPEATS regions of `steps` calls of fn(i), each bracketed by events on the current stream; returns the region
    times in ms.  Every region starts from a drained device."""
    times = []
    i = first
    for _ in range(REPEATS):
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record()
        for _ in range(steps):
            fn(i)
            i += 1
        stop.record()
        torch.cuda.synchronize()
        times.append(start.elapsed_time(stop))
    return times


def run_linear(args, rdk, torch, w, vocab, batch, mode_name, path, steps, warmup, traffic):
    """Times `steps` passes of redistribution (mode_name) + verification over the batch; returns the figures."""
    bias, kept, E = vocab
    B = batch["z_p"].shape[0]
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
        p, q_hat = prob_inputs(batch, kept)
        p_host, q_host, kind = torch.from_numpy(p), torch.from_numpy(q_hat), "prob"
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
    rdk.rdk_timing_select("*")
    for i in range(20):
        step(i)
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    per_kernel = {}
    for nm in KERNEL_NAMES:
        cnt, ms = rdk.rdk_timing_read(nm)
        if cnt:
            per_kernel[nm] = {"launches_per_step": cnt / 20.0, "avg_us": 1e3 * ms / cnt}
    dominant = max((k for k in per_kernel if k != "sequence_scan_kernel"),
                   key=lambda k: per_kernel[k]["avg_us"] * per_kernel[k]["launches_per_step"])
    print("kernels of one %s step:" % mode_name, {k: round(v["avg_us"], 1) for k, v in per_kernel.items()}, file=sys.stderr)

    # the timed regions: K steps each, the dominant kernel's launches bracketed by events on the launch stream
    rdk.rdk_timing_select(dominant + "/8")             # every eighth launch: an event pair per launch would slow the step
    regions = timed_regions(torch, step, steps, warmup)
    rdk.rdk_timing_select(None)
    cnt, kms = rdk.rdk_timing_read(dominant)
    total_ms = float(np.median(regions))
    ms_per_step = total_ms / steps

    kk = (max(w.k, 1) + 15) // 16 * 16
    esz = 2 if w.logits_bf16 else 4
    alg = algorithmic_bytes(dominant, w, B, kk, fused, esz)
    avg_s = kms / cnt * 1e-3
    achieved = alg / avg_s / 1e9
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic.get((w.name, mode_name, path, dominant)),
                "avg_launch_us": round(avg_s * 1e6, 2),
                "algorithmic_bytes_per_launch": alg}
    if dominant == "sparse_product_kernel":
        roofline["limited_by"] = "line gathers through the vector L1 (extra.sparse_gather), not HBM: the fraction is the algorithmic HBM bytes over the peak"
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
    if fused and args.in_flight > 1:
        # context, not the metric (opt-in: overlapping launches would blur the per-kernel averages of a profile): two batches in flight on two streams (own outputs and workspaces), so that the
        # latency-bound end of one batch's step overlaps the streaming start of the next one's
        streams = [torch.cuda.Stream() for _ in range(2)]
        vouts2 = [rdk.VerifyOutputs(B, w.N, w.gamma, dev) for _ in range(2)]

        def step2(i):
            with torch.cuda.stream(streams[i % 2]):
                rdk.rdk_redistribute_verify(kern, mode, ps[i % C], qs[i % C], seed=2506, offset=i * B, gamma=w.gamma,
                                            p_kind=kind, q_kind=kind, outputs=vouts2[i % 2])

        K2 = max(400, steps)
        for i in range(20):
            step2(i)
        els = []
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(K2):
                step2(i)
            torch.cuda.synchronize()
            els.append(time.perf_counter() - t0)
        el = float(np.median(els))
        res_extra["two_batches_in_flight"] = {"streams": 2, "steps": K2, "ms_per_step": round(el / K2 * 1e3, 5),
                                              "positions_per_s": round(K2 * B / el, 1), "clock": "host, drained device on both sides, median of 3"}
    return {"ms_per_step": ms_per_step, "value": B / (ms_per_step * 1e-3), "roofline": roofline, **res_extra,
            "region_ms": [round(t, 4) for t in regions],
            "kernels": {k: {"avg_us": round(v["avg_us"], 2), "per_step": v["launches_per_step"]} for k, v in per_kernel.items()},
            "step_algorithmic_GBs": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
            "step_frac_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "kernel_build_s": round(build_s, 3),
            "accept_rate": float(vout.accept.float().mean().item()), "mean_alpha": float(vout.alpha.mean().item())}


def linear_leg(args, rdk, torch, w, vocab, batch, mode, steps, traffic):
    """One fused linear form on a workload, boiled down for `extra`."""
    o = run_linear(args, rdk, torch, w, vocab, batch, mode, "fused", steps, 10, traffic)
    leg = {"mode": mode, "path": "fused", "positions_per_s": round(o["value"], 1), "ms_per_step": round(o["ms_per_step"], 5),
           "roofline": o["roofline"], "kernels": o["kernels"], "step_frac_of_hbm_peak": o["step_frac_of_hbm_peak"]}
    for key in ("sparse_gather", "two_batches_in_flight"):
        if key in o:
            leg[key] = o[key]
    return leg


def run_draft(args, rdk, torch, w, vocab, batch, steps):
    """Draft-side sampling alone: rdk_sample_draft with the top-k sparse kernel, q' never materialised."""
    bias, kept, E = vocab
    dev = torch.device("cuda:0")
    kern = rdk.rdk_build_kernel(w.N, torch.from_numpy(kept).to(dev), rdk.SPARSE_TOPK, embeddings=torch.from_numpy(E).to(dev),
                                tau=w.tau, k=w.k)
    if w.logits_bf16:
        q_host, kind = torch.from_numpy(batch["z_q"]).to(torch.bfloat16), "logit"
    else:
        q_host, kind = torch.from_numpy(prob_inputs(batch, kept)[1]), "prob"
    qs = [q_host.to(dev) for _ in range(max(1, args.copies))]
    ids = torch.empty(w.B, dtype=torch.int32, device=dev)
    qd = torch.empty(w.B, dtype=torch.float32, device=dev)
    call = lambda i: rdk.rdk_sample_draft(kern, qs[i % len(qs)], 2506, i * w.B, kind, draft_ids=ids, q_draft=qd)
    for i in range(5):
        call(i)
    ms = float(np.median(timed_regions(torch, call, steps, 5))) / steps
    return {"entry": "rdk_sample_draft (sparse top-k, no target row)", "ms_per_step": round(ms, 5),
            "positions_per_s": round(w.B / (ms * 1e-3), 1)}


def run_multi(args, rdk, torch, w, vocab, batch, steps, traffic, C=4):
    """Several candidates per position (rdk_verify_multi) on the materialised rows of the sparse form: the candidates
    drawn from q', then one pass over p and q' per rejected candidate."""
    bias, kept, E = vocab
    dev = torch.device("cuda:0")
    kern = rdk.rdk_build_kernel(w.N, torch.from_numpy(kept).to(dev), rdk.SPARSE_TOPK, embeddings=torch.from_numpy(E).to(dev),
                                tau=w.tau, k=w.k)
    if w.logits_bf16:
        p_host, q_host, kind = torch.from_numpy(batch["z_p"]).to(torch.bfloat16), torch.from_numpy(batch["z_q"]).to(torch.bfloat16), "logit"
    else:
        p, q_hat = prob_inputs(batch, kept)
        p_host, q_host, kind = torch.from_numpy(p), torch.from_numpy(q_hat), "prob"
    n_copies = max(1, args.copies)
    ps = [p_host.to(dev) for _ in range(n_copies)]
    qp = [rdk.rdk_redistribute_linear(kern, rdk.LINEAR_SPARSE, q_host.to(dev), kind) for _ in range(n_copies)]
    out = rdk.MultiOutputs(w.B, C, dev)
    call = lambda i: rdk.rdk_verify_multi(ps[i % n_copies], qp[i % n_copies], C, 2506, i * w.B, kind, outputs=out)
    for i in range(5):
        call(i)
    torch.cuda.synchronize()
    rdk.rdk_timing_select("verify_multi_kernel")
    ms = float(np.median(timed_regions(torch, call, steps, 5))) / steps
    rdk.rdk_timing_select(None)
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
                         "traffic": traffic.get((w.name, "multi", "C%d" % C, "verify_multi_kernel")),
                         "avg_launch_us": round(kms / cnt * 1e3, 2), "algorithmic_bytes_per_launch": alg}}


def run_exact(rdk, torch, w, vocab, batch, fmt, calls, traffic):
    """Exact dense redistribution (Alg. 1 with the full M): the 16-bit matrix-core contraction at N=256000, n=32000, B=512
    (bound by the matrix cores), or the fp32 one at N=32000, n=8000, B=64 (three bf16 parts per operand on the bf16
    matrix cores: bound by streaming M from HBM once)."""
    bias, kept, E = vocab
    dev = torch.device("cuda:0")
    kern = rdk.rdk_build_kernel(w.N, torch.from_numpy(kept).to(dev), rdk.DENSE_BF16 if fmt == "bf16" else rdk.DENSE_F32,
                                embeddings=torch.from_numpy(E).to(dev), tau=w.tau)
    q = torch.from_numpy(prob_inputs(batch, kept)[1]).to(dev)
    out = torch.empty((w.B, w.N), dtype=torch.float32, device=dev)
    call = lambda i: rdk.rdk_redistribute_exact(kern, q, out=out)
    for i in range(2):
        call(i)
    torch.cuda.synchronize()
    kname = "exact_bf16_kernel" if fmt == "bf16" else "exact_f32_split_kernel"
    rdk.rdk_timing_select(kname)
    ms_call = float(np.median(timed_regions(torch, call, calls, 0))) / calls
    rdk.rdk_timing_select(None)
    cnt, kms = rdk.rdk_timing_read(kname)
    flops = 2.0 * w.B * w.n * w.N
    k_tf = flops / (kms / cnt * 1e-3) / 1e12
    row_err = float((out.double().sum(1) - 1).abs().max().item())
    esz = 2 if fmt == "bf16" else 4
    del kern, out, q
    torch.cuda.empty_cache()
    tr = traffic.get((w.name, "exact", fmt, kname))
    if fmt == "bf16":
        roofline = {"kernel": kname, "bound": "mfma", "achieved": round(k_tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(k_tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": tr,
                    "avg_launch_us": round(kms / cnt * 1e3, 1), "algorithmic_flops_per_launch": flops,
                    "operands": "M rounded to bf16, drafter rows to 11 bits, both fed as scaled fp16 (same matrix-core rate as bf16)"}
    else:
        # M read once, the drafter rows read once, the output written once (the split partials are not counted)
        alg = 4.0 * w.n * w.N + 4.0 * w.B * (w.n + w.N)
        gbs = alg / (kms / cnt * 1e-3) / 1e9
        roofline = {"kernel": kname, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": tr, "avg_launch_us": round(kms / cnt * 1e3, 1),
                    "algorithmic_bytes_per_launch": alg, "algorithmic_TFLOPs": round(k_tf, 1),
                    "fp32_matrix_peak_TFLOPs": MFMA_F32_PEAK_TFLOPS}
    return {"workload": "%s: N=%d n=%d B=%d, M %s %.2f GB" % (w.name, w.N, w.n, w.B, fmt, esz * w.n * w.N / 1e9),
            "ms_per_call": round(ms_call, 3), "positions_per_s": round(w.B / (ms_call * 1e-3), 1), "roofline": roofline,
            "call_TFLOPs": round(flops / (ms_call * 1e-3) / 1e12, 1), "max_row_sum_error": row_err}


def workload_inputs(synth, name):
    w = synth.WORKLOADS[name]
    bias, kept, E, rng = synth.make_vocab(w)
    return w, (bias, kept, E), synth.make_batch(w, bias, kept, rng)


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
    ap.add_argument("--in-flight", type=int, default=1, help="2: also time two batches in flight on two streams (extra.two_batches_in_flight)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle baseline")
    ap.add_argument("--no-extra", action="store_true", help="skip the other forms and workloads")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="budget of each of the two oracle timings")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this library runs on one GPU (positions are independent: shard the batch); run with --gpus 1")

    import torch
    from paper_2506_03206_amd import rdk, synth

    wname = args.workload or "llama3"
    torch.cuda.set_device(0)
    traffic, traffic_note = measured_traffic()

    # Yardstick for hardware byte counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE): one elementwise pass that
    # reads exactly 256 MiB and writes exactly 256 MiB; it is the only launch with 2^26 float elements.
    cal = torch.zeros(1 << 26, dtype=torch.float32, device="cuda:0")
    cal_out = torch.empty_like(cal)
    torch.add(cal, 1.0, out=cal_out)
    torch.cuda.synchronize()
    del cal, cal_out
    torch.cuda.empty_cache()

    t0 = time.time()
    w, vocab, batch = workload_inputs(synth, wname)
    if not w.logits_bf16:
        prob_inputs(batch, vocab[1])
    gen_s = time.time() - t0
    B = w.B

    r = run_linear(args, rdk, torch, w, vocab, batch, args.mode, args.path, args.steps, args.warmup, traffic)
    extra = {k: r[k] for k in ("kernels", "region_ms", "step_algorithmic_GBs", "step_frac_of_hbm_peak", "kernel_build_s",
                               "accept_rate", "mean_alpha")}
    extra["timing"] = "median of %d regions of %d steps" % (REPEATS, args.steps)
    extra["traffic_source"] = traffic_note if traffic else (traffic_note or "no counter figures on file")
    extra["input_gen_s"] = round(gen_s, 2)
    for key in ("sparse_gather", "two_batches_in_flight"):
        if key in r:
            extra[key] = r[key]
    if not args.no_extra:
        other = "taylor" if args.mode == "sparse" else "sparse"
        torch.cuda.empty_cache()
        extra["other_linear_form"] = linear_leg(args, rdk, torch, w, vocab, batch, other, max(20, args.steps // 2), traffic)
        extra["draft_sampling"] = run_draft(args, rdk, torch, w, vocab, batch, max(20, args.steps // 2))
        extra["multi_candidate"] = run_multi(args, rdk, torch, w, vocab, batch, max(20, args.steps // 4), traffic)
        torch.cuda.empty_cache()
        # N=32000, n=8000, B=64: the exact fp32 product and both fused linear forms
        w1, vocab1, batch1 = workload_inputs(synth, "n32k")
        extra["n32k"] = {"exact_f32": run_exact(rdk, torch, w1, vocab1, batch1, "f32", 20, traffic),
                         "sparse": linear_leg(args, rdk, torch, w1, vocab1, batch1, "sparse", 50, traffic),
                         "taylor": linear_leg(args, rdk, torch, w1, vocab1, batch1, "taylor", 50, traffic)}
        extra["exact_f32"] = extra["n32k"]["exact_f32"]
        del batch1
        # N=151936, n=16384, B=1024, bf16 logits, k=32: both fused forms
        w3, vocab3, batch3 = workload_inputs(synth, "qwen_extreme")
        extra["qwen_extreme"] = {"sparse": linear_leg(args, rdk, torch, w3, vocab3, batch3, "sparse", 10, traffic),
                                 "taylor": linear_leg(args, rdk, torch, w3, vocab3, batch3, "taylor", 20, traffic)}
        del batch3
        torch.cuda.empty_cache()
        # N=256000, n=32000, B=512: the exact 16-bit product, and the linear forms on the same inputs
        w4, vocab4, batch4 = workload_inputs(synth, "dense256k")
        extra["exact_bf16"] = run_exact(rdk, torch, w4, vocab4, batch4, "bf16", 10, traffic)
        extra["dense256k_linear"] = {"sparse": linear_leg(args, rdk, torch, w4, vocab4, batch4, "sparse", 20, traffic),
                                     "taylor": linear_leg(args, rdk, torch, w4, vocab4, batch4, "taylor", 20, traffic)}
        del batch4
        torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(args, w, batch, vocab[1])

    line = {"metric": "redistribute+verify positions/sec at N=%d, n=%d" % (w.N, w.n), "value": round(r["value"], 1),
            "unit": "positions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(r["ms_per_step"], 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": "%s: N=%d n=%d B=%d (%d seqs x %d drafts) k=%d, %s linear RDK + verify/sample, %s inputs"
                       % (w.name, w.N, w.n, B, w.seqs, w.gamma, w.k, args.mode, "bf16 logit" if w.logits_bf16 else "fp32 prob"),
                       "mode": args.mode, "path": args.path, "N": w.N, "n": w.n, "B": B, "k": w.k},
            "roofline": r["roofline"], "cpu_baseline": cpu, "extra": extra}
    print(json.dumps(line))


# ---- the oracle on the host: one thread, and one worker process per core over blocks of positions
_CPU = {}


def _cpu_rows(task):
    """The oracle pipeline on rows [b0, b1) of the batch (TLI -> redistribution -> accept / residual / sample)."""
    import oracle
    b0, b1, offset = task
    w, mode = _CPU["w"], _CPU["mode"]
    if w.logits_bf16:
        pr = oracle.probs_from(_CPU["z_p"][b0:b1], "logit")
        qr = oracle.probs_from(_CPU["z_q"][b0:b1], "logit")
    else:
        pr, qr = _CPU["p"][b0:b1], _CPU["q_hat"][b0:b1]
    if mode == "sparse":
        qp = oracle.redistribute_batch("sparse", qr, _CPU["kept"], w.N, sparse=_CPU["sparse"])
    else:
        qp = oracle.redistribute_batch("taylor", qr, _CPU["kept"], w.N, p=pr)
    oracle.verify_batch(pr, qp, 2506, offset + b0, gamma=w.gamma if (b1 - b0) % w.gamma == 0 else 0)
    return b1 - b0


def cpu_baseline(args, w, batch, kept):
    """The oracle, as it stands, on the host: same pipeline, same batch, for about cpu_seconds on one thread and again
    with one worker process per host core (blocks of eight positions handed out in order)."""
    import multiprocessing as mp
    from paper_2506_03206_amd import synth
    B = w.B
    _CPU.update(w=w, mode=args.mode, kept=kept)
    if w.logits_bf16:
        _CPU.update(z_p=batch["z_p"], z_q=batch["z_q"])
    else:
        p, q_hat = prob_inputs(batch, kept)
        _CPU.update(p=p, q_hat=q_hat)
    if args.mode == "sparse":
        # a kernel of the same shape from raw draws (random neighbours, unnormalised weights): the oracle's own top-k
        # construction is O(N n d) in fp64, minutes at this size, and the time of the redistribution does not depend on
        # the values
        idx, a = synth.random_neighbour_draws(np.random.default_rng(1), w.N, kept, w.k)
        _CPU["sparse"] = (idx, a, np.ones(kept.size))
    blocks = [(b0, min(B, b0 + 8)) for b0 in range(0, B, 8)]
    # one thread
    rows, t0, rep = 0, time.time(), 0
    while time.time() - t0 < args.cpu_seconds:
        for b0, b1 in blocks:
            rows += _cpu_rows((b0, b1, rep * B))
            if time.time() - t0 >= args.cpu_seconds:
                break
        rep += 1
    el1 = time.time() - t0
    single = rows / el1
    # one worker per core (fork: the batch is shared, not copied)
    cores = os.cpu_count() or 1
    usable = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else cores
    workers = max(1, min(usable, 64))
    rounds = max(1, int(round(single * args.cpu_seconds * workers / B)))       # whole passes over the batch
    tasks = [(b0, b1, r * B) for r in range(rounds) for b0, b1 in blocks]
    ctx = mp.get_context("fork")
    with ctx.Pool(workers) as pool:
        pool.map(_cpu_rows, [(0, 1, 0)] * workers)                             # workers up, library loaded
        t0 = time.time()
        done = sum(pool.imap_unordered(_cpu_rows, tasks, chunksize=1))
        el2 = time.time() - t0
    return {"value": round(done / el2, 1), "unit": "positions/s", "cores": workers, "kind": "oracle",
            "host_cpu_count": cores, "usable_cores": usable,
            "single_thread": {"value": round(single, 1), "unit": "positions/s", "cores": 1, "positions": rows, "seconds": round(el1, 1)},
            "sample": "%d positions (%d passes over the same batch; TLI -> %s redistribution -> accept/residual/sample, fp64) in "
                      "%.1f s on %d worker processes; single thread: %d positions in %.1f s; the sparse kernel is a "
                      "random-neighbour kernel of the same shape" % (done, rounds, args.mode, el2, workers, rows, el1)}


if __name__ == "__main__":
    main()
