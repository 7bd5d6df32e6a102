"""The entry point that allocates nothing (rdk_verify_sample_static): its outputs against rdk_verify_sample's on the
same inputs, bit for bit, on two calls in a row of which the second is smaller (the scratch array keeps the first
call's contents), and the refusal of a batch beyond the fixed scratch size."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_03206_amd import synth
from parity_util import check_verify_outputs

pytestmark = pytest.mark.gpu

FIELDS = ("draft_ids", "accept", "alpha", "resid_mass", "resid_ids", "n_accepted", "out_tokens")


def inputs(N, B, seed, logits):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 3, size=(2, B, N)).astype(np.float32)
    e = np.exp(z.astype(np.float64) - z.max(2, keepdims=True))
    p, q = [(x / x.sum(2 if x.ndim == 3 else 1, keepdims=True)) for x in (e[0], e[1])]
    p_in = z[0] if logits else p.astype(np.float32)
    return p_in, q.astype(np.float32)


def test_static_scratch_entry_point_matches_workspace_entry_point():
    from paper_2506_03206_amd import rdk
    rdk.lib()
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    # first a batch of 5000-id rows (5 block sums per row), then a smaller one that leaves most of the scratch stale
    for (N, B, gamma, logits, seed) in ((5000, 24, 4, True, 1), (1300, 6, 3, False, 2)):
        p_in, q = inputs(N, B, seed, logits)
        kind = "logit" if logits else "prob"
        p_d, q_d = torch.from_numpy(p_in).to(dev), torch.from_numpy(q).to(dev)
        ref = rdk.rdk_verify_sample(p_d, q_d, seed=11, offset=3, gamma=gamma, p_kind=kind)
        out = rdk.VerifyOutputs(B, N, gamma, dev)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rdk.rdk_verify_sample_static(p_d, q_d, seed=11, offset=3, gamma=gamma, p_kind=kind, outputs=out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for name in FIELDS:
            assert torch.equal(getattr(out, name), getattr(ref, name)), (name, N, B)
        # and both agree with the oracle
        p64 = oracle.probs_from(p_in, kind)
        q64 = q.astype(np.float64)
        check_verify_outputs(out, oracle.verify_batch(p64, q64, 11, 3, gamma=gamma), p64, q64, 11, 3, gamma, kind, min_exact=0.9)
    # the bonus draw (no drafter row) through the same entry point
    p_in, _ = inputs(1300, 6, 3, False)
    p_d = torch.from_numpy(p_in).to(dev)
    ref = rdk.rdk_verify_sample(p_d, None, seed=5)
    out = rdk.VerifyOutputs(6, 1300, 0, dev)
    rdk.rdk_verify_sample_static(p_d, None, seed=5, outputs=out)
    assert torch.equal(out.resid_ids, ref.resid_ids) and torch.equal(out.resid_mass, ref.resid_mass)


def test_static_scratch_entry_point_refuses_large_batches():
    from paper_2506_03206_amd import rdk
    dev = torch.device("cuda:0")
    N, B = 1024 * 40, 4096                       # 3 * 4 * B * 40 bytes of block sums = 1.9 MB ... doubled below
    p = torch.zeros((2, N), dtype=torch.float32, device=dev)
    # the size check happens on the host before anything is launched: rows are never read, so a 2-row tensor with a
    # declared batch of 3 * B positions (5.9 MB of block sums) is enough to ask for too much
    import ctypes
    d = rdk.VerifyDesc(B=3 * B, N=N, gamma=0, sample_draft=1, seed=0, offset=0)
    ids = torch.zeros(3 * B, dtype=torch.int32, device=dev)
    acc = torch.zeros(3 * B, dtype=torch.uint8, device=dev)
    rc = rdk.lib().rdk_verify_sample_static(ctypes.byref(d), ctypes.c_void_p(p.data_ptr()), rdk.PROB_F32, N,
                                            ctypes.c_void_p(p.data_ptr()), N, ctypes.c_void_p(ids.data_ptr()),
                                            ctypes.c_void_p(acc.data_ptr()), None, None, ctypes.c_void_p(ids.data_ptr()),
                                            None, None, None)
    assert rc == 6                               # RDK_ERR_WORKSPACE
