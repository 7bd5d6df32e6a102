"""Shared helpers of the GPU parity tests: tolerances, and validity checks for sampled ids."""
import numpy as np

# fp32 paths: |g - o| <= RTOL |o| + ATOL elementwise; bf16 dense path: RTOL_BF16.
RTOL, ATOL = 1e-5, 1e-7
RTOL_BF16 = 2e-3
# A sampled id is compared exactly unless the threshold lies within CDF_TOL * total of a step of the
# prefix sum: there fp32 summation order may pick the neighbour, which is accepted if it is valid.
CDF_TOL = 1e-5


def assert_close(g, o, rtol=RTOL, atol=ATOL, what=""):
    g, o = np.asarray(g, dtype=np.float64), np.asarray(o, dtype=np.float64)
    assert g.shape == o.shape, (g.shape, o.shape)
    assert np.all(np.isfinite(g)), what + ": non-finite values"
    err = np.abs(g - o) - (rtol * np.abs(o) + atol)
    if err.max() > 0:
        i = np.unravel_index(np.argmax(err), err.shape)
        raise AssertionError("%s: worst element %s gpu=%.9g oracle=%.9g (rel %.3g)" %
                             (what, i, g[i], o[i], abs(g[i] - o[i]) / max(abs(o[i]), 1e-300)))


def check_sampled_ids(weights, u, gpu_ids, oracle_ids, tol=CDF_TOL, what=""):
    """weights [B,N] fp64 (the oracle's), u [B], ids from both sides.  Returns the number of exact matches."""
    exact = 0
    for b in range(weights.shape[0]):
        g, o = int(gpu_ids[b]), int(oracle_ids[b])
        if g == o:
            exact += 1
            continue
        c = np.cumsum(weights[b])
        total = c[-1]
        assert total > 0 and 0 <= g < weights.shape[1], "%s row %d: gpu id %d, oracle id %d" % (what, b, g, o)
        thr = u[b] * total
        margin = min(abs(thr - c[o]), abs(thr - (c[o - 1] if o > 0 else 0.0)))
        assert margin <= tol * total, "%s row %d: ids differ (gpu %d, oracle %d) with margin %.3g of the total" % (
            what, b, g, o, margin / total)
        # the gpu id must be what the oracle's rule gives for a threshold moved by at most tol * total
        assert weights[b, g] > 0, "%s row %d: gpu id %d has zero weight" % (what, b, g)
        assert c[g] > thr - tol * total and (g == 0 or c[g - 1] <= thr + tol * total), (what, b, g, o)
    return exact
