#!/usr/bin/env python3
"""Acceptance rate against pruning level on synthetic heavy-tailed targets (the experiment of Sec. 5.2,
"Acceptance recovery"), run through the device library.

Target logits are Student-t (5 degrees of freedom) noise on a Zipf rank bias; the drafter sees the target logits
plus unit Gaussian noise and keeps only the n most frequent ids (frequency-ranked pruning).  Per pruning level the
mean acceptance rate alpha = sum_j min(p_j, q'_j) (Def. 2.1) of three schemes is printed:
  masked  -- the drafter's probabilities on the kept ids, not renormalised (pruning without redistribution),
  tli     -- token-level intersection, Eq. 1,
  taylor  -- the first-order RDK form, Eq. 3.
The paper does not give its generator's parameters, so the numbers are context for its figure, not a reproduction.

  python -m paper_2506_03206_amd.acceptance_sweep [--N 200000] [--B 64] [--keep 100000 20000 5000 2000 500]
"""
import argparse
import json

import numpy as np


def make_inputs(N, B, sigma, zipf_s, seed):
    """Target / drafter logits [B, N] (fp32) and the ids ordered by falling expected frequency."""
    rng = np.random.default_rng(seed)
    rank_of = rng.permutation(N)                                   # rank of each id; ranks are scattered over the ids
    bias = (-zipf_s * np.log1p(rank_of)).astype(np.float32)
    z_p = (sigma * rng.standard_t(5, size=(B, N))).astype(np.float32) + bias[None, :]
    z_d = z_p + rng.standard_normal((B, N), dtype=np.float32)
    return z_p, z_d, np.argsort(rank_of, kind="stable").astype(np.int32)


def sweep(N=200000, B=64, keep=(100000, 20000, 5000, 2000, 500), sigma=2.0, zipf_s=1.0, seed=0, device="cuda:0"):
    """Every number below comes out of the library: torch only holds the buffers and picks columns.

    The softmax of a logit row is the library's redistribution with the identity kernel over the whole vocabulary
    (every id kept); a pruned drafter is its logits on the kept ids (the softmax over them is Eq. 1 applied to the full
    softmax); the overlap of two sub-distributions on the kept ids is rdk_verify_sample on those columns."""
    import torch
    from . import rdk
    z_p, z_d, by_frequency = make_inputs(N, B, sigma, zipf_s, seed)
    dev = torch.device(device)
    zp, zd = torch.from_numpy(z_p).to(dev), torch.from_numpy(z_d).to(dev)
    everything = rdk.rdk_build_kernel(N, torch.arange(N, dtype=torch.int32, device=dev), rdk.IDENTITY)
    p_full = rdk.rdk_redistribute_linear(everything, rdk.LINEAR_SPARSE, zp, "logit")      # softmax(z_p)
    q_full = rdk.rdk_redistribute_linear(everything, rdk.LINEAR_SPARSE, zd, "logit")      # softmax(z_d)
    rows = []
    for n in keep:
        kept = np.sort(by_frequency[:n])
        kept_d = torch.from_numpy(kept).to(dev)
        cols = kept_d.long()
        kern = rdk.rdk_build_kernel(N, kept_d, rdk.IDENTITY)
        zq = zd[:, cols].contiguous()                               # what the pruned drafter head emits
        # (a) masked only: the drafter's full-vocabulary probabilities on the kept ids, no renormalisation; its overlap
        #     with the target is the sum of min(p, q) over the kept columns
        a_masked = rdk.rdk_verify_sample(p_full[:, cols].contiguous(), q_full[:, cols].contiguous(), seed=1, offset=0,
                                         gamma=0).alpha
        # (b) token-level intersection: the identity kernel
        tli = rdk.rdk_redistribute_linear(kern, rdk.LINEAR_SPARSE, zq, "logit")
        a_tli = rdk.rdk_verify_sample(zp, tli, seed=1, offset=0, gamma=0, p_kind="logit").alpha
        # (c) Eq. 3, fused with the verification
        a_taylor = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_TAYLOR, zp, zq, seed=1, offset=0, gamma=0,
                                               p_kind="logit", q_kind="logit").alpha
        rows.append({"N": N, "n": int(n), "kept_fraction": n / N, "alpha_masked": float(a_masked.mean()),
                     "alpha_tli": float(a_tli.mean()), "alpha_taylor": float(a_taylor.mean())})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--N", type=int, default=200000)
    ap.add_argument("--B", type=int, default=64)
    ap.add_argument("--keep", type=int, nargs="+", default=[100000, 20000, 5000, 2000, 500])
    ap.add_argument("--sigma", type=float, default=2.0)
    ap.add_argument("--zipf", type=float, default=1.0)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    for row in sweep(args.N, args.B, args.keep, args.sigma, args.zipf, args.seed):
        print(json.dumps(row))


if __name__ == "__main__":
    main()
