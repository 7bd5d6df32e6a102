"""Seeded synthetic inputs for the RDK redistribute + verify path.

This module only *makes inputs*: target / drafter logits and probabilities with a
long-tailed (Zipf) token bias, a kept-id set that imitates frequency-ranked
pruning, and Gaussian token embeddings that stand in for the affinity statistics.
It holds none of the method's arithmetic (no softmax, no normalisation of a kernel:
logits and raw draws only) and imports neither the GPU library nor the CPU oracle,
so both can be fed from it.

Shapes and value distributions follow what section 5.1 of the paper reports for real
models: a long-tailed token distribution (a small share of the ids carries almost
all of the mass), per-position logit standard deviations of 2-4, and peaked
output probabilities.  Real corpora and model weights are replaced by these
draws everywhere.

Draw order for a given seed (numpy PCG64): id permutation -> kept set ->
embeddings -> target noise -> drafter noise.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int            # target vocabulary |T|
    n: int            # kept ids |I| (drafter vocabulary after pruning)
    seqs: int         # sequences
    gamma: int        # draft tokens per sequence; positions B = seqs * gamma
    sigma: float      # std of the Gaussian part of the target logits
    zipf_s: float     # exponent of the rank bias  -s * ln(rank)
    d: int            # embedding width
    tau: float        # temperature of Eq. 2
    k: int            # neighbours per pruned id in the sparse kernel
    kept_rule: str    # "uniform" | "top_ranks"  (top ranks + 10 % random)
    logits_bf16: bool = False
    seed: int = 0

    @property
    def B(self):
        return self.seqs * self.gamma


WORKLOADS = {
    # small enough for the oracle to run every path in full
    "tiny": Workload("tiny", 1024, 256, 4, 4, 2.0, 1.1, 64, 0.1, 8, "uniform"),
    "n32k": Workload("n32k", 32000, 8000, 8, 8, 2.0, 1.1, 128, 0.1, 16, "top_ranks"),
    # Llama-3-sized vocabulary: the headline workload
    "llama3": Workload("llama3", 128256, 32064, 32, 8, 3.0, 1.0, 128, 0.1, 16, "top_ranks"),
    "qwen_extreme": Workload("qwen_extreme", 151936, 16384, 128, 8, 3.0, 1.05, 256, 0.05, 32, "top_ranks",
                             logits_bf16=True),
    "dense256k": Workload("dense256k", 256000, 32000, 64, 8, 3.0, 1.0, 256, 0.1, 16, "top_ranks"),
}


def scaled(w, **kw):
    """A copy of a workload with some fields replaced (used for reduced test sizes)."""
    from dataclasses import replace
    return replace(w, **kw)


def bf16_round(x):
    """Round fp32 to the nearest bf16 (ties to even); returned as fp32 holding bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x):
    """The 16-bit patterns of fp32 values that are already exact bf16 numbers."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def make_vocab(w: Workload, rng=None):
    """Rank bias over ids, the kept-id set (ascending int32) and the embeddings [N,d] fp32."""
    rng = rng or np.random.default_rng(w.seed)
    perm = rng.permutation(w.N)                     # rank of id j is 1 + perm[j]
    bias = (-w.zipf_s * np.log(1.0 + perm)).astype(np.float32)
    if w.kept_rule == "uniform":
        kept = rng.choice(w.N, size=w.n, replace=False)
    elif w.kept_rule == "top_ranks":
        n_top = (9 * w.n) // 10
        by_rank = np.argsort(perm, kind="stable")   # ids in order of rank
        rest = by_rank[n_top:]
        extra = rng.choice(rest.size, size=w.n - n_top, replace=False)
        kept = np.concatenate([by_rank[:n_top], rest[extra]])
    else:
        raise ValueError(w.kept_rule)
    kept = np.sort(kept).astype(np.int32)
    E = rng.standard_normal((w.N, w.d), dtype=np.float32)
    return bias, kept, E, rng


def make_batch(w: Workload, bias, kept, rng, B=None):
    """Target and drafter logits for B positions (draws only; whoever wants probabilities applies its own softmax).

    Returns a dict with
      z_p [B,N] fp32 target logits,
      z_d [B,N] fp32 the drafter's logits over the whole vocabulary (the target's plus unit Gaussian noise),
      z_q [B,n] fp32 = z_d on the kept slots (what a pruned drafter head emits).
    With logits_bf16 the logits are bf16 values (held in fp32).
    """
    B = B or w.B
    n = kept.size
    out = {"z_p": np.empty((B, w.N), np.float32), "z_d": np.empty((B, w.N), np.float32), "z_q": np.empty((B, n), np.float32)}
    for r0 in range(0, B, 16):                       # 16 rows at a time: target noise, then drafter noise
        r1 = min(B, r0 + 16)
        z_p = rng.standard_normal((r1 - r0, w.N), dtype=np.float32) * np.float32(w.sigma) + bias[None, :]
        z_d = z_p + rng.standard_normal((r1 - r0, w.N), dtype=np.float32)   # the drafter sees a noisy target
        if w.logits_bf16:
            z_p, z_d = bf16_round(z_p), bf16_round(z_d)
        out["z_p"][r0:r1] = z_p
        out["z_d"][r0:r1] = z_d
        out["z_q"][r0:r1] = z_d[:, kept]
    return out


def make(w: Workload, B=None):
    """Vocabulary + one batch for a workload."""
    bias, kept, E, rng = make_vocab(w)
    batch = make_batch(w, bias, kept, rng, B)
    batch.update(kept_ids=kept, E=E, bias=bias)
    return batch


def random_neighbour_draws(rng, N, kept, k):
    """The raw material of a top-k-shaped kernel, draws only: for each pruned id k distinct kept slots drawn uniformly
    (nbr_idx [N-n,k] int32) and a positive unnormalised affinity per entry (fp64, as small as real ones).  Turning them
    into a row-stochastic kernel (Eq. 2 over the retained entries) is left to the caller."""
    n = kept.size
    P = N - n
    idx = rng.integers(0, n, size=(P, k), dtype=np.int32)
    while k > 1:                                     # redraw the few rows that hold a slot twice
        srt = np.sort(idx, axis=1)
        dup = np.nonzero((srt[:, 1:] == srt[:, :-1]).any(axis=1))[0]
        if dup.size == 0:
            break
        idx[dup] = rng.integers(0, n, size=(dup.size, k), dtype=np.int32)
    a = np.exp(-5.0 - 3.0 * rng.random((P, k)))
    return idx, a
