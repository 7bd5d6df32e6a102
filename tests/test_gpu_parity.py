"""GPU parity: every entry point of the C-ABI library against the CPU oracle, element by element, on
seeded inputs small enough for the oracle yet spanning several tiles and a ragged tail."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2506_03206_amd import synth
from parity_util import (ATOL, RTOL, RTOL_DENSE, RTOL_DENSE_UNROUNDED, assert_close, check_multi, check_sampled_ids,
                         check_verify_outputs, make_inputs, operand_round_M, operand_round_q, random_row_stochastic,
                         random_trees, stochastic_topk_kernel)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rdk():
    from paper_2506_03206_amd import rdk as mod
    mod.lib()
    assert torch.cuda.is_available()
    return mod


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def bf16_tensor(x):
    """fp32 array holding exact bf16 values -> torch bf16 tensor on the device."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).cuda()


@pytest.fixture(scope="module")
def tiny():
    w = synth.WORKLOADS["tiny"]
    data = make_inputs(w)
    data["w"] = w
    data["sparse"] = oracle.build_sparse(data["E"], data["kept_ids"], w.tau, w.k)
    data["dense"] = oracle.build_dense(data["E"], data["kept_ids"], w.tau)
    return data


# ragged sizes: N not a multiple of 4 (scalar paths), of 1024 (partial block), n odd, B not a multiple of 16
RAGGED = synth.scaled(synth.WORKLOADS["tiny"], name="ragged", N=3001, n=517, seqs=7, gamma=3, k=5, d=24, seed=3)


@pytest.fixture(scope="module")
def ragged():
    data = make_inputs(RAGGED)
    data["w"] = RAGGED
    data["sparse"] = oracle.build_sparse(data["E"], data["kept_ids"], RAGGED.tau, RAGGED.k)
    data["dense"] = oracle.build_dense(data["E"], data["kept_ids"], RAGGED.tau)
    return data


# --------------------------------------------------------------------------------------------- Philox
def test_philox_stream_matches_oracle(rdk):
    seed, offset, count = 0xDEADBEEFCAFEF00D, (1 << 32) - 300, 1000
    words = rdk.rdk_philox_words(seed, offset, count).cpu().numpy().view(np.uint32)
    for i in list(range(0, count, 37)) + [299, 300, 301, count - 1]:
        idx = offset + i
        ref = oracle.philox4x32_10([idx & 0xFFFFFFFF, idx >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        assert words[i].tolist() == ref.tolist()


# --------------------------------------------------------------------------------------------- kernel construction
@pytest.mark.parametrize("case", ["tiny", "ragged"])
def test_build_sparse_matches_oracle(rdk, tiny, ragged, case):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.SPARSE_TOPK, embeddings=dev(data["E"]), tau=w.tau, k=w.k)
    idx, wt, sw = [t.cpu().numpy() for t in rdk.rdk_kernel_get_sparse(kern)]
    o_idx, o_w, o_sw = data["sparse"]
    assert np.array_equal(idx, o_idx)            # neighbour sets and their order (fp64 affinities on both sides)
    assert_close(wt, o_w, what="neighbour weights")
    assert_close(sw, o_sw, what="diagonal weights")


@pytest.mark.parametrize("case", ["tiny", "ragged"])
def test_build_dense_matches_oracle(rdk, tiny, ragged, case):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.DENSE_F32, embeddings=dev(data["E"]), tau=w.tau)
    M = rdk.rdk_kernel_get_dense(kern).cpu().numpy()
    assert_close(M, data["dense"], what="dense M")
    assert np.abs(M.astype(np.float64).sum(1) - 1).max() < 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_features_from_scores_and_kernel_from_data(rdk, ragged, dtype):
    """Omega estimated from data (Sec. 3): centred token features from sampled target logits, then the top-k kernel
    built from them, against the oracle's features and the oracle's kernel."""
    w = ragged["w"]
    T = 70
    rng = np.random.default_rng(21)
    z = (rng.normal(size=(T, 24)) @ rng.normal(size=(24, w.N)) + rng.normal(size=w.N)[None, :]).astype(np.float32)
    if dtype == "bf16":
        z = synth.bf16_round(z)
        z_dev = bf16_tensor(z)
    else:
        z_dev = dev(z)
    F = rdk.rdk_features_from_scores(z_dev)
    ref_F = oracle.features_from_scores(z)
    assert_close(F.cpu().numpy(), ref_F, rtol=1e-5, atol=2e-6, what="centred features")
    kern = rdk.rdk_build_kernel(w.N, dev(ragged["kept_ids"]), rdk.SPARSE_TOPK, embeddings=F, tau=w.tau, k=w.k)
    idx, wt, sw = [t.cpu().numpy() for t in rdk.rdk_kernel_get_sparse(kern)]
    o_idx, o_w, o_sw, om = oracle.build_sparse(F.cpu().numpy(), ragged["kept_ids"], w.tau, w.k, return_affinities=True)
    # neighbour lists agree wherever the oracle's ranking is not a near-tie (both sides start from the same fp32 features)
    clear = np.min(-np.diff(om, axis=1), axis=1) > 1e-9
    assert clear.mean() > 0.99 and np.array_equal(idx[clear], o_idx[clear])
    if clear.all():
        assert_close(wt, o_w, what="neighbour weights")
        assert_close(sw, o_sw, what="diagonal weights")


def test_build_validation(rdk, tiny):
    w = tiny["w"]
    bad = tiny["kept_ids"].copy()
    bad[[3, 4]] = bad[[4, 3]]
    with pytest.raises(rdk.RdkError) as e:
        rdk.rdk_build_kernel(w.N, dev(bad), rdk.IDENTITY)
    assert e.value.status == 4
    M = tiny["dense"].astype(np.float32).copy()
    M[5] *= 1.01
    with pytest.raises(rdk.RdkError) as e:
        rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.DENSE_F32, dense_M=dev(M))
    assert e.value.status == 5
    idx, wt, sw = tiny["sparse"]
    with pytest.raises(rdk.RdkError) as e:
        rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.SPARSE_TOPK, k=w.k,
                             sparse=(dev(idx), dev(wt * 1.5, torch.float32), dev(sw, torch.float32)))
    assert e.value.status == 5


# --------------------------------------------------------------------------------------------- redistribution
def oracle_rows(data, mode, q_kind="prob", p_kind="prob", kernel=None):
    w = data["w"]
    q = data["q_hat"] if q_kind == "prob" else oracle.probs_from(data["z_q"], "logit")
    p = data["p"] if p_kind == "prob" else oracle.probs_from(data["z_p"], "logit")
    return oracle.redistribute_batch(mode, q, data["kept_ids"], w.N, p=p, M=kernel if mode == "exact" else None,
                                     sparse=kernel if mode == "sparse" else None)


@pytest.mark.parametrize("case", ["tiny", "ragged"])
@pytest.mark.parametrize("q_kind", ["prob", "logit"])
def test_sparse_redistribution(rdk, tiny, ragged, case, q_kind):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    idx, wt, sw = data["sparse"]
    wt32, sw32 = wt.astype(np.float32), sw.astype(np.float32)     # both sides use the same stored kernel
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.SPARSE_TOPK, k=w.k,
                                sparse=(dev(idx), dev(wt32), dev(sw32)))
    q = dev(data["q_hat"]) if q_kind == "prob" else dev(data["z_q"])
    out = rdk.rdk_redistribute_linear(kern, rdk.LINEAR_SPARSE, q, q_kind).cpu().numpy()
    ref = oracle_rows(data, "sparse", q_kind, kernel=(idx, wt32, sw32))
    assert_close(out, ref, what="sparse q'")
    assert np.abs(out.astype(np.float64).sum(1) - 1).max() < 1e-5


@pytest.mark.parametrize("case", ["tiny", "ragged"])
@pytest.mark.parametrize("kinds", [("prob", "prob"), ("logit", "logit"), ("prob", "logit")])
def test_taylor_redistribution(rdk, tiny, ragged, case, kinds):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    p_kind, q_kind = kinds
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.IDENTITY)
    q = dev(data["q_hat"]) if q_kind == "prob" else dev(data["z_q"])
    p = dev(data["p"]) if p_kind == "prob" else dev(data["z_p"])
    out = rdk.rdk_redistribute_linear(kern, rdk.LINEAR_TAYLOR, q, q_kind, p=p, p_kind=p_kind).cpu().numpy()
    ref = oracle_rows(data, "taylor", q_kind, p_kind)
    assert_close(out, ref, what="Eq. 3")


def test_taylor_bf16_logits(rdk, tiny):
    w = tiny["w"]
    zp, zq = synth.bf16_round(tiny["z_p"]), synth.bf16_round(tiny["z_q"])
    kern = rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.IDENTITY)
    out = rdk.rdk_redistribute_linear(kern, rdk.LINEAR_TAYLOR, bf16_tensor(zq), "logit", p=bf16_tensor(zp),
                                      p_kind="logit").cpu().numpy()
    ref = oracle.redistribute_batch("taylor", oracle.probs_from(zq, "logit"), tiny["kept_ids"], w.N,
                                    p=oracle.probs_from(zp, "logit"))
    assert_close(out, ref, what="Eq. 3, bf16 logits")


@pytest.mark.parametrize("case", ["tiny", "ragged"])
def test_identity_kernel_is_tli(rdk, tiny, ragged, case):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.IDENTITY)
    ref = oracle_rows(data, "tli")
    for fn in (lambda: rdk.rdk_redistribute_exact(kern, dev(data["q_hat"])),
               lambda: rdk.rdk_redistribute_linear(kern, rdk.LINEAR_SPARSE, dev(data["q_hat"]))):
        assert_close(fn().cpu().numpy(), ref, what="identity kernel")


@pytest.mark.parametrize("case", ["tiny", "ragged"])
@pytest.mark.parametrize("q_kind", ["prob", "logit"])
def test_exact_fp32(rdk, tiny, ragged, case, q_kind):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    M32 = data["dense"].astype(np.float32)
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.DENSE_F32, dense_M=dev(M32))
    q = dev(data["q_hat"]) if q_kind == "prob" else dev(data["z_q"])
    out = rdk.rdk_redistribute_exact(kern, q, q_kind).cpu().numpy()
    ref = oracle_rows(data, "exact", q_kind, kernel=M32)
    assert_close(out, ref, what="exact fp32")


def test_exact_fp32_keeps_every_part(rdk, ragged):
    """The fp32 product runs on three bf16 parts per operand.  Two cases in which a dropped or mispaired part shows
    at once: a one-hot drafter row must return the kernel row bit for bit (the parts of an fp32 number add up to it
    exactly), and a kernel that sends each slot to its own id must return the normalised drafter row to fp32
    rounding (losing the trailing part of the drafter weights would cost 2^-16 of each value)."""
    w = ragged["w"]
    M32 = ragged["dense"].astype(np.float32)
    kern = rdk.rdk_build_kernel(w.N, dev(ragged["kept_ids"]), rdk.DENSE_F32, dense_M=dev(M32))
    slots = [0, 1, 7, 8, 15, 16, 255, 256, w.n - 2, w.n - 1] + list(range(20, 20 + 60))   # 70 rows: two row groups
    q = np.zeros((len(slots), w.n), dtype=np.float32)
    q[np.arange(len(slots)), slots] = 1.0
    out = rdk.rdk_redistribute_exact(kern, dev(q)).cpu().numpy()
    assert np.array_equal(out, M32[slots]), "one-hot rows must reproduce the kernel rows exactly"

    P = np.zeros((w.n, w.N), dtype=np.float32)
    P[np.arange(w.n), ragged["kept_ids"]] = 1.0
    kern = rdk.rdk_build_kernel(w.N, dev(ragged["kept_ids"]), rdk.DENSE_F32, dense_M=dev(P))
    rng = np.random.default_rng(11)
    q = (rng.random((9, w.n)) * np.exp(rng.normal(0.0, 3.0, size=(9, w.n)))).astype(np.float32)   # full mantissas, wide range
    out = rdk.rdk_redistribute_exact(kern, dev(q)).cpu().numpy()
    for b in range(q.shape[0]):
        ref = oracle.tli(q[b])
        got = out[b, ragged["kept_ids"]].astype(np.float64)
        assert np.max(np.abs(got - ref) / ref) < 5e-7, "row %d: %.3e" % (b, np.max(np.abs(got - ref) / ref))
        assert np.count_nonzero(out[b]) == w.n


@pytest.mark.parametrize("case", ["tiny", "ragged"])
def test_exact_bf16(rdk, tiny, ragged, case):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    M32 = data["dense"].astype(np.float32)
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.DENSE_BF16, dense_M=dev(M32))
    Mb = operand_round_M(M32)                    # the kernel as stored: bf16 values (zero below 2^-29)
    assert np.array_equal(rdk.rdk_kernel_get_dense(kern).cpu().numpy().astype(np.float64), Mb)
    assert np.array_equal(Mb[Mb >= 2.0 ** -29], synth.bf16_round(M32).astype(np.float64)[Mb >= 2.0 ** -29])
    out = rdk.rdk_redistribute_exact(kern, dev(data["q_hat"])).cpu().numpy()
    # tight: fp64 on the same rounded operands, rows rescaled to unit mass
    ref, ref_stored = np.empty((w.B, w.N)), np.empty((w.B, w.N))
    for b in range(w.B):
        qt = oracle.tli(data["q_hat"][b])
        r = oracle.redistribute_dense(operand_round_q(qt), Mb)
        ref[b] = r / r.sum()
        r = oracle.redistribute_dense(qt, Mb)
        ref_stored[b] = r / r.sum()
    assert_close(out, ref, rtol=2e-5, atol=ATOL, what="exact bf16 vs rounded operands")
    # the stated tolerance of the dense path: the drafter rows as given, the kernel as stored
    assert_close(out, ref_stored, rtol=RTOL_DENSE, atol=ATOL, what="exact bf16 vs the stored kernel")
    # and against the kernel before it was rounded to its storage format
    assert_close(out, oracle_rows(data, "exact", kernel=M32), rtol=RTOL_DENSE_UNROUNDED, atol=ATOL, what="exact bf16 vs fp32 kernel")
    assert np.abs(out.astype(np.float64).sum(1) - 1).max() < 1e-5


@pytest.mark.parametrize("B", [130, 300, 530])
def test_exact_bf16_batch_shapes(rdk, ragged, B):
    """The dense bf16 product picks its workgroup shape from the batch size: one case per shape, the largest
    spanning two rows of workgroups with a ragged last one."""
    w = ragged["w"]
    M32 = ragged["dense"].astype(np.float32)
    kern = rdk.rdk_build_kernel(w.N, dev(ragged["kept_ids"]), rdk.DENSE_BF16, dense_M=dev(M32))
    # Rows of integer counts c / 2^15 with c <= 255 and sum(c) = 2^15: every value and every partial sum is exact in
    # bf16 and fp32, so the rounding of the normalised row to bf16 cannot fall on different sides of a tie on the
    # two sides (a flipped dominant slot would move an output by half a bf16 ulp, far beyond the tolerance).
    rng = np.random.default_rng(100 + B)
    c = rng.integers(0, 128, size=(B, w.n))
    for b in range(B):
        order = rng.permutation(w.n)
        diff, t = (1 << 15) - int(c[b].sum()), 0
        while diff != 0:
            i, step = order[t % w.n], (1 if diff > 0 else -1)
            if 0 <= c[b, i] + step <= 255:
                c[b, i] += step
                diff -= step
            t += 1
    c[0] = 0
    c[0, w.n // 2] = 1 << 15                                     # a one-hot row
    q = (c / float(1 << 15)).astype(np.float32)
    assert np.all(q.sum(1, dtype=np.float64) == 1.0) and np.array_equal(synth.bf16_round(q), q)
    out = rdk.rdk_redistribute_exact(kern, dev(q)).cpu().numpy()
    Mb = operand_round_M(M32)
    ref = np.empty((B, w.N))
    for b in range(B):
        qb = operand_round_q(oracle.tli(q[b]))
        r = oracle.redistribute_dense(qb, Mb)
        ref[b] = r / r.sum()
    assert_close(out, ref, rtol=2e-5, atol=ATOL, what="exact bf16, B=%d" % B)


# --------------------------------------------------------------------------------------------- verification
def run_verify_case(rdk, p_in, p_kind, p64, qp32, gamma, seed, offset, draft_ids=None):
    o = rdk.rdk_verify_sample(p_in, None if qp32 is None else dev(qp32), seed, offset, gamma, p_kind,
                              draft_ids=None if draft_ids is None else dev(draft_ids))
    torch.cuda.synchronize()
    q64 = None if qp32 is None else qp32.astype(np.float64)
    ref = oracle.verify_batch(p64, q64, seed, offset, sample_draft=draft_ids is None, draft_ids=draft_ids, gamma=gamma)
    check_verify_outputs(o, ref, p64, q64, seed, offset, gamma, p_kind)
    if q64 is not None and p_kind == "prob":      # identical fp32 inputs on both sides: the accept flags must agree exactly
        same = o.draft_ids.cpu().numpy() == ref["draft_ids"]
        assert np.array_equal(o.accept.cpu().numpy()[same], ref["accept"][same])
    return o, ref


@pytest.mark.parametrize("case", ["tiny", "ragged"])
def test_verify_prob_inputs(rdk, tiny, ragged, case):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    idx, wt, sw = data["sparse"]
    qp = oracle_rows(data, "sparse", kernel=(idx, wt, sw)).astype(np.float32)
    p64 = data["p"].astype(np.float64)
    run_verify_case(rdk, dev(data["p"]), "prob", p64, qp, w.gamma, seed=11, offset=5)
    run_verify_case(rdk, dev(data["p"]), "prob", p64, qp, 0, seed=12, offset=(1 << 40))
    # caller-supplied drafts, including an out-of-range one
    drafts = np.arange(w.B, dtype=np.int32) * 7 % w.N
    drafts[1] = -1
    run_verify_case(rdk, dev(data["p"]), "prob", p64, qp, w.gamma, seed=13, offset=0, draft_ids=drafts)
    # bonus draw
    run_verify_case(rdk, dev(data["p"]), "prob", p64, None, 0, seed=14, offset=9)


def test_verify_logit_inputs(rdk, tiny):
    w = tiny["w"]
    qp = oracle_rows(tiny, "taylor").astype(np.float32)
    p64 = oracle.probs_from(tiny["z_p"], "logit")
    run_verify_case(rdk, dev(tiny["z_p"]), "logit", p64, qp, w.gamma, seed=21, offset=0)
    zb = synth.bf16_round(tiny["z_p"])
    run_verify_case(rdk, bf16_tensor(zb), "logit", oracle.probs_from(zb, "logit"), qp, w.gamma, seed=22, offset=0)


def test_verify_degenerate_rows(rdk):
    """alpha = 1 (no residual), point masses, zero-probability drafts, long sequences (gamma > 16)."""
    N, B = 2500, 40
    rng = np.random.default_rng(5)
    p = rng.gamma(0.3, size=(B, N)).astype(np.float32)
    p[:, rng.choice(N, 800, replace=False)] = 0
    p = (p / p.sum(1, keepdims=True)).astype(np.float32)
    q = p.copy()                       # rows 0..9: q' == p -> alpha = 1, residual mass 0, resid id -1
    q[10:20] = 0
    q[10:20, 1234] = 1.0               # point-mass drafter
    q[20:] = np.roll(p[20:], 17, axis=1)
    o, ref = run_verify_case(rdk, dev(p), "prob", p.astype(np.float64), q, 20, seed=31, offset=0)
    assert (o.resid_ids.cpu().numpy()[:10] == -1).all() and (ref["resid_ids"][:10] == -1).all()
    assert o.accept.cpu().numpy()[:10].all()
    assert (o.draft_ids.cpu().numpy()[10:20] == 1234).all()


@pytest.mark.parametrize("p_kind", ["prob", "logit", "bf16"])
def test_verify_large_batch(rdk, p_kind):
    """From 128 positions on every row is finished by a workgroup of its own (a quarter of a 1024-id block per
    wavefront): ragged N with a short last block, drawn and caller-supplied drafts, and the same finish on q' of Eq. 3
    when the fused call also writes the rows out."""
    w = synth.scaled(synth.WORKLOADS["tiny"], name="manyrows", N=5003, n=1201, seqs=26, gamma=5, seed=23)
    data = make_inputs(w)
    kept = data["kept_ids"]
    if p_kind == "prob":
        p_in, p_dev = data["p"], dev(data["p"])
    elif p_kind == "logit":
        p_in, p_dev = data["z_p"], dev(data["z_p"])
    else:
        p_in = synth.bf16_round(data["z_p"])
        p_dev = bf16_tensor(p_in)
    kind = "prob" if p_kind == "prob" else "logit"
    p64 = oracle.probs_from(p_in, kind)
    q64 = data["q_hat"].astype(np.float64)
    ref_qp = oracle.redistribute_batch("taylor", q64, kept, w.N, p=p64)
    qp32 = ref_qp.astype(np.float32)
    run_verify_case(rdk, p_dev, kind, p64, qp32, w.gamma, seed=61, offset=7)
    drafts = (np.arange(w.B, dtype=np.int32) * 977) % w.N
    drafts[3] = w.N                                              # out of range: never accepted
    run_verify_case(rdk, p_dev, kind, p64, qp32, w.gamma, seed=62, offset=0, draft_ids=drafts)
    ki = rdk.rdk_build_kernel(w.N, dev(kept), rdk.IDENTITY)
    rows = torch.empty(w.B, w.N, device="cuda")
    o = rdk.rdk_redistribute_verify(ki, rdk.LINEAR_TAYLOR, p_dev, dev(data["q_hat"]), 63, 1, w.gamma, kind, q_prime=rows)
    assert_close(rows.cpu().numpy(), ref_qp, what="q' of the fused call")
    check_verify_outputs(o, oracle.verify_batch(p64, ref_qp, 63, 1, gamma=w.gamma), p64, ref_qp, 63, 1, w.gamma, kind)


def test_fused_sparse_very_large_vocab(rdk):
    """The sparse form sums per 64-id block; above 262144 ids a row has more block sums than the finish keeps in registers
    (64 per lane), and they are re-read from memory when the crossings are located.  Drawn and caller-supplied drafts."""
    w = synth.scaled(synth.WORKLOADS["tiny"], name="widevocab", N=300017, n=3001, k=5, seqs=2, gamma=4, seed=17)
    data = make_inputs(w)
    kept = data["kept_ids"]
    idx, wt, sw = stochastic_topk_kernel(np.random.default_rng(4), w.N, kept, w.k)
    wt32, sw32 = wt.astype(np.float32), sw.astype(np.float32)
    kern = rdk.rdk_build_kernel(w.N, dev(kept), rdk.SPARSE_TOPK, k=w.k, sparse=(dev(idx), dev(wt32), dev(sw32)))
    p64 = data["p"].astype(np.float64)
    ref_qp = oracle.redistribute_batch("sparse", data["q_hat"].astype(np.float64), kept, w.N, sparse=(idx, wt32, sw32))
    seed, offset = 71, 4
    o = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_SPARSE, dev(data["p"]), dev(data["q_hat"]), seed, offset, w.gamma)
    check_verify_outputs(o, oracle.verify_batch(p64, ref_qp, seed, offset, gamma=w.gamma), p64, ref_qp, seed, offset, w.gamma, "prob")
    drafts = (np.arange(w.B, dtype=np.int32) * 50021) % w.N
    o = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_SPARSE, dev(data["p"]), dev(data["q_hat"]), seed, offset, w.gamma,
                                    draft_ids=dev(drafts))
    ref = oracle.verify_batch(p64, ref_qp, seed, offset, sample_draft=False, draft_ids=drafts, gamma=w.gamma)
    check_verify_outputs(o, ref, p64, ref_qp, seed, offset, w.gamma, "prob")
    d, qd = rdk.rdk_sample_draft(kern, dev(data["q_hat"]), seed, offset)
    u0 = np.array([oracle.uniforms(seed, offset + b)[0] for b in range(w.B)])
    ref_d = np.array([oracle.sample_cdf(ref_qp[b], u0[b]) for b in range(w.B)])
    check_sampled_ids(ref_qp, u0, d.cpu().numpy(), ref_d, what="draft from q'")


def test_verify_very_large_vocab(rdk):
    """More 1024-id blocks per row than a wavefront keeps in registers (N > 2^19): the block partials are then
    re-read from memory when the prefix-sum crossings are located."""
    N, B = 600011, 6
    rng = np.random.default_rng(9)
    z = rng.normal(0, 3, size=(2, B, N))
    e = np.exp(z - z.max(2, keepdims=True))
    p, q = [(x / x.sum(1, keepdims=True)).astype(np.float32) for x in e]
    run_verify_case(rdk, dev(p), "prob", p.astype(np.float64), q, 3, seed=41, offset=2)
    drafts = (np.arange(B, dtype=np.int32) * 50021) % N
    run_verify_case(rdk, dev(p), "prob", p.astype(np.float64), q, 3, seed=42, offset=0, draft_ids=drafts)
    # several candidates per position at the same size: 586 block sums per row in LDS, ten per lane
    p64, q64 = p.astype(np.float64), q.astype(np.float64)
    ref = oracle.verify_multi_batch(p64, q64, 3, 43, 7)
    o = rdk.rdk_verify_multi(dev(p), dev(q), 3, 43, 7)
    for i in range(3):
        us = np.array([oracle.multi_uniform(43, 7 + b, i) for b in range(B)])
        check_sampled_ids(q64, us, o.cand_ids.cpu().numpy()[:, i], ref["cand_ids"][:, i], what="candidate %d" % i)
    o = rdk.rdk_verify_multi(dev(p), dev(q), 3, 43, 7, cand_ids=dev(ref["cand_ids"]))
    check_multi(o, ref, p64, q64, 43, 7, 3, min_exact=0.5)


def test_pipeline_end_to_end(rdk, tiny):
    """rdk_build_kernel -> rdk_redistribute_linear -> rdk_verify_sample on the device vs the oracle chain."""
    w = tiny["w"]
    kern = rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.SPARSE_TOPK, embeddings=dev(tiny["E"]), tau=w.tau, k=w.k)
    qp = rdk.rdk_redistribute_linear(kern, rdk.LINEAR_SPARSE, dev(tiny["q_hat"]))
    o = rdk.rdk_verify_sample(dev(tiny["p"]), qp, seed=77, offset=0, gamma=w.gamma)
    ref_qp = oracle_rows(tiny, "sparse", kernel=tiny["sparse"])
    assert_close(qp.cpu().numpy(), ref_qp, what="q' from the device-built kernel")
    ref = oracle.verify_batch(tiny["p"], ref_qp, 77, 0, gamma=w.gamma)
    assert_close(o.alpha.cpu().numpy(), ref["alpha"], what="alpha")
    us = np.array([oracle.uniforms(77, b) for b in range(w.B)])
    check_sampled_ids(ref_qp, us[:, 0], o.draft_ids.cpu().numpy(), ref["draft_ids"], what="draft")


def test_entry_points_reject_bad_arguments(rdk, tiny):
    """Every redistribute / verify entry point checks its arguments on the host and returns a status without
    launching anything: NULL, a leading dimension shorter than the row, a misaligned pointer, a short workspace,
    a form the kernel does not offer."""
    import ctypes
    w = tiny["w"]
    L = rdk.lib()
    q, p = dev(tiny["q_hat"]), dev(tiny["p"])
    out = torch.empty((w.B, w.N), dtype=torch.float32, device="cuda")
    ident = rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.IDENTITY)
    ws = ident.workspace(w.B)
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    lin = lambda **kw: L.rdk_redistribute_linear(*[kw.get(k, v) for k, v in dict(
        kernel=ident.handle, mode=rdk.LINEAR_TAYLOR, p=P(p), p_kind=rdk.PROB_F32, ldp=w.N, q=P(q), q_kind=rdk.PROB_F32, ldq=w.n,
        B=w.B, out=P(out), ldo=w.N, ws=P(ws), ws_bytes=ws.numel(), stream=st).items()])
    assert lin() == 0
    assert lin(out=None) == 1 and lin(q=None) == 1 and lin(p=None) == 1
    assert lin(ldo=w.N - 1) == 2 and lin(ldq=w.n - 1) == 2 and lin(ldp=w.N - 4) == 2 and lin(B=0) == 2
    assert lin(q_kind=9) == 3 and lin(mode=5) == 3
    assert lin(ws_bytes=64) == 6
    assert lin(q=ctypes.c_void_p(q.data_ptr() + 4)) == 9 and lin(out=ctypes.c_void_p(out.data_ptr() + 8)) == 9
    dense = rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.DENSE_F32, dense_M=dev(tiny["dense"].astype(np.float32)))
    dws = dense.workspace(w.B)
    assert lin(kernel=dense.handle, mode=rdk.LINEAR_SPARSE, ws=P(dws), ws_bytes=dws.numel()) == 7   # no sparse product with a dense kernel
    idx, wt, sw = tiny["sparse"]
    sparse = rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.SPARSE_TOPK, k=w.k,
                                  sparse=(dev(idx), dev(wt, torch.float32), dev(sw, torch.float32)))
    sws = sparse.workspace(w.B)
    assert L.rdk_redistribute_exact(sparse.handle, P(q), rdk.PROB_F32, w.n, w.B, P(out), w.N, P(sws), sws.numel(), st) == 7
    torch.cuda.synchronize()


def test_acceptance_sweep_matches_oracle(rdk):
    """The Sec. 5.2 sweep (masked / TLI / Eq. 3 acceptance against pruning level) at a small size against the oracle."""
    from paper_2506_03206_amd import acceptance_sweep as sw
    N, B, keep = 6000, 8, (3000, 600, 60)
    rows = sw.sweep(N=N, B=B, keep=keep, seed=4)
    z_p, z_d, by_frequency = sw.make_inputs(N, B, 2.0, 1.0, 4)
    p64 = oracle.probs_from(z_p, "logit")
    q_full = oracle.probs_from(z_d, "logit")
    for row, n in zip(rows, keep):
        kept = np.sort(by_frequency[:n])
        q_hat = q_full[:, kept]
        masked = np.zeros((B, N))
        masked[:, kept] = q_hat
        a_masked = np.mean([oracle.overlap(p64[b], masked[b])[0] for b in range(B)])
        tli = oracle.redistribute_batch("tli", q_hat, kept, N)
        a_tli = np.mean([oracle.overlap(p64[b], tli[b])[0] for b in range(B)])
        tay = oracle.redistribute_batch("taylor", q_hat, kept, N, p=p64)
        a_tay = np.mean([oracle.overlap(p64[b], tay[b])[0] for b in range(B)])
        # every softmax and every sum ran in the library; the means of eight rows carry the stated tolerance
        for name, ref_a in (("alpha_masked", a_masked), ("alpha_tli", a_tli), ("alpha_taylor", a_tay)):
            assert abs(row[name] - ref_a) <= RTOL * ref_a + ATOL, (name, n, row[name], ref_a)
        assert row["alpha_tli"] >= row["alpha_masked"] - 1e-6          # Eq. 1 only scales the kept mass up


# --------------------------------------------------------------------------------------------- draft-side sampling
@pytest.mark.parametrize("case", ["tiny", "ragged"])
@pytest.mark.parametrize("form", ["sparse", "sparse_rows", "identity", "dense_f32", "dense_bf16"])
def test_sample_draft(rdk, tiny, ragged, case, form):
    """rdk_sample_draft: ids drawn from q' alone (no target row) against the oracle's inverse CDF of its own q'."""
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    idx, wt, sw = data["sparse"]
    wt32, sw32 = wt.astype(np.float32), sw.astype(np.float32)
    qp = torch.zeros((w.B, w.N), dtype=torch.float32, device="cuda")
    if form in ("sparse", "sparse_rows"):
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.SPARSE_TOPK, k=w.k, sparse=(dev(idx), dev(wt32), dev(sw32)))
        ref_qp = oracle_rows(data, "sparse", kernel=(idx, wt32, sw32))
    elif form == "identity":
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.IDENTITY)
        ref_qp = oracle_rows(data, "tli")
    elif form == "dense_f32":
        M32 = data["dense"].astype(np.float32)
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.DENSE_F32, dense_M=dev(M32))
        ref_qp = oracle_rows(data, "exact", kernel=M32)
    else:   # bf16 storage: the reference rows are the product of the rounded operands, rescaled to unit mass
        M32 = data["dense"].astype(np.float32)
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.DENSE_BF16, dense_M=dev(M32))
        Mb = operand_round_M(M32)
        ref_qp = np.empty((w.B, w.N))
        for b in range(w.B):
            r = oracle.redistribute_dense(operand_round_q(oracle.tli(data["q_hat"][b])), Mb)
            ref_qp[b] = r / r.sum()
    rtol = 4e-5 if form == "dense_bf16" else RTOL
    seed, offset = 909, (1 << 35) + 3
    d, qd = rdk.rdk_sample_draft(kern, dev(data["q_hat"]), seed, offset, q_prime=None if form == "sparse" else qp)
    torch.cuda.synchronize()
    d, qd = d.cpu().numpy(), qd.cpu().numpy()
    u0 = np.array([oracle.uniforms(seed, offset + b)[0] for b in range(w.B)])
    ref_d = np.array([oracle.sample_cdf(ref_qp[b], u0[b]) for b in range(w.B)])
    assert check_sampled_ids(ref_qp, u0, d, ref_d, tol=4e-5 if form == "dense_bf16" else 1e-5, what="draft from q'") >= 0.9 * w.B
    assert_close(qd, ref_qp[np.arange(w.B), d], rtol=rtol, what="q' at the drafted id")
    if form != "sparse":
        assert_close(qp.cpu().numpy(), ref_qp, rtol=rtol, what="rows written on the way")
    if form in ("sparse", "sparse_rows"):   # the fused verification draws the same ids from the same block sums
        o = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_SPARSE, dev(data["p"]), dev(data["q_hat"]), seed, offset, w.gamma)
        assert np.array_equal(o.draft_ids.cpu().numpy(), d)
        # and verifying these ids afterwards accepts exactly where the oracle does
        o2 = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_SPARSE, dev(data["p"]), dev(data["q_hat"]), seed, offset, w.gamma,
                                         draft_ids=dev(d))
        p64 = data["p"].astype(np.float64)
        ref = oracle.verify_batch(p64, ref_qp, seed, offset, sample_draft=False, draft_ids=d, gamma=w.gamma)
        assert np.array_equal(o2.accept.cpu().numpy(), ref["accept"])


def test_sample_draft_zero_row_and_errors(rdk, tiny):
    w = tiny["w"]
    kern = rdk.rdk_build_kernel(w.N, dev(tiny["kept_ids"]), rdk.IDENTITY)
    with pytest.raises(rdk.RdkError) as e:                      # rows must be written somewhere for this kernel
        rdk.rdk_sample_draft(kern, dev(tiny["q_hat"]), 1, 0)
    assert e.value.status == 1


def test_extreme_rows(rdk, ragged):
    """Rows at the edges of the input domain through both fused forms: a one-hot target, a target disjoint from the
    drafter's support (alpha = 0), drafter rows that are mostly exact zeros, and logits spanning +-60."""
    w = ragged["w"]
    idx, wt, sw = ragged["sparse"]
    wt32, sw32 = wt.astype(np.float32), sw.astype(np.float32)
    kept = ragged["kept_ids"]
    B = 8
    rng = np.random.default_rng(77)
    p = rng.gamma(0.2, size=(B, w.N)).astype(np.float32)
    q = rng.gamma(0.2, size=(B, w.n)).astype(np.float32)
    p[0] = 0
    p[0, kept[5]] = 1.0                                   # one-hot target on a kept id
    p[1] = 0
    is_kept = np.zeros(w.N, dtype=bool)
    is_kept[kept] = True
    p[1, np.nonzero(~is_kept)[0][::7]] = 1.0              # target mass only on pruned ids
    q[2, 10:] = 0                                         # drafter mass on ten slots
    q[3] = 0
    q[3, w.n - 1] = 3.0                                   # a single slot, not normalised
    p = (p / p.sum(1, keepdims=True)).astype(np.float32)
    p64 = p.astype(np.float64)
    ks = rdk.rdk_build_kernel(w.N, dev(kept), rdk.SPARSE_TOPK, k=w.k, sparse=(dev(idx), dev(wt32), dev(sw32)))
    ki = rdk.rdk_build_kernel(w.N, dev(kept), rdk.IDENTITY)
    for kern, gmode, mode, sparse in ((ks, rdk.LINEAR_SPARSE, "sparse", (idx, wt32, sw32)), (ki, rdk.LINEAR_TAYLOR, "taylor", None)):
        qp = torch.empty((B, w.N), dtype=torch.float32, device="cuda")
        o = rdk.rdk_redistribute_verify(kern, gmode, dev(p), dev(q), 5, 0, 4, q_prime=qp)
        ref_qp = oracle.redistribute_batch(mode, q, kept, w.N, p=p64, sparse=sparse)
        assert_close(qp.cpu().numpy(), ref_qp, what="q' (%s), extreme rows" % mode)
        ref = oracle.verify_batch(p64, ref_qp, 5, 0, gamma=4)
        check_verify_outputs(o, ref, p64, ref_qp, 5, 0, 4, "prob", min_exact=0.75)
    # logits over a wide range, fp32 and bf16
    z_p = (rng.normal(size=(B, w.N)) * 20).clip(-60, 60).astype(np.float32)
    z_q = (rng.normal(size=(B, w.n)) * 20).clip(-60, 60).astype(np.float32)
    for zp_dev, zq_dev, zp, zq in ((dev(z_p), dev(z_q), z_p, z_q),
                                   (bf16_tensor(synth.bf16_round(z_p)), bf16_tensor(synth.bf16_round(z_q)),
                                    synth.bf16_round(z_p), synth.bf16_round(z_q))):
        pl, ql = oracle.probs_from(zp, "logit"), oracle.probs_from(zq, "logit")
        qp = torch.empty((B, w.N), dtype=torch.float32, device="cuda")
        o = rdk.rdk_redistribute_verify(ki, rdk.LINEAR_TAYLOR, zp_dev, zq_dev, 6, 3, 4, "logit", "logit", q_prime=qp)
        ref_qp = oracle.redistribute_batch("taylor", ql, kept, w.N, p=pl)
        assert_close(qp.cpu().numpy(), ref_qp, what="Eq. 3, wide logits")
        ref = oracle.verify_batch(pl, ref_qp, 6, 3, gamma=4)
        check_verify_outputs(o, ref, pl, ref_qp, 6, 3, 4, "logit", min_exact=0.75)


def test_drafter_row_without_mass(rdk, ragged):
    """Eq. 1 is undefined for a drafter row whose kept slots carry no mass: the oracle refuses it, and every
    redistribution of the library returns the zero row (one contract for all forms), so that the verification of
    such a position sees alpha = 0, residual mass = sum p, no draft, no acceptance, and draws its token from p."""
    w = ragged["w"]
    kept = ragged["kept_ids"]
    idx, wt, sw = ragged["sparse"]
    wt32, sw32 = wt.astype(np.float32), sw.astype(np.float32)
    M32 = ragged["dense"].astype(np.float32)
    B, zero_rows = 6, (1, 4)
    q = ragged["q_hat"][:B].copy()
    q[list(zero_rows)] = 0
    p = ragged["p"][:B]
    p64 = p.astype(np.float64)
    with pytest.raises(ValueError):
        oracle.tli(q[1])
    live = [b for b in range(B) if b not in zero_rows]
    ks = rdk.rdk_build_kernel(w.N, dev(kept), rdk.SPARSE_TOPK, k=w.k, sparse=(dev(idx), dev(wt32), dev(sw32)))
    ki = rdk.rdk_build_kernel(w.N, dev(kept), rdk.IDENTITY)
    kf = rdk.rdk_build_kernel(w.N, dev(kept), rdk.DENSE_F32, dense_M=dev(M32))
    kb = rdk.rdk_build_kernel(w.N, dev(kept), rdk.DENSE_BF16, dense_M=dev(M32))
    forms = {
        "sparse": (lambda: rdk.rdk_redistribute_linear(ks, rdk.LINEAR_SPARSE, dev(q)), dict(mode="sparse", sparse=(idx, wt32, sw32))),
        "taylor": (lambda: rdk.rdk_redistribute_linear(ki, rdk.LINEAR_TAYLOR, dev(q), p=dev(p)), dict(mode="taylor", p=p64)),
        "identity": (lambda: rdk.rdk_redistribute_exact(ki, dev(q)), dict(mode="tli")),
        "exact fp32": (lambda: rdk.rdk_redistribute_exact(kf, dev(q)), dict(mode="exact", M=M32)),
        "exact bf16": (lambda: rdk.rdk_redistribute_exact(kb, dev(q)), None),
    }
    for name, (run, ref_args) in forms.items():
        out = run().cpu().numpy()
        assert np.isfinite(out).all(), name
        for b in zero_rows:
            assert not out[b].any(), "%s: row %d must be the zero row" % (name, b)
        if ref_args is not None:      # the other rows are untouched by their neighbours
            mode = ref_args.pop("mode")
            ref = oracle.redistribute_batch(mode, q[live], kept, w.N, **{k: (v[live] if k == "p" else v) for k, v in ref_args.items()})
            assert_close(out[live], ref, what=name + ", rows with mass")
        else:
            assert np.abs(out[live].astype(np.float64).sum(1) - 1).max() < 1e-5
    # the fused calls and the draft draw on the same batch
    us = np.array([oracle.uniforms(9, b) for b in range(B)])
    for kern, gmode in ((ks, rdk.LINEAR_SPARSE), (ki, rdk.LINEAR_TAYLOR)):
        o = rdk.rdk_redistribute_verify(kern, gmode, dev(p), dev(q), 9, 0, 0)
        for b in zero_rows:
            assert o.draft_ids[b].item() == -1 and o.accept[b].item() == 0 and o.alpha[b].item() == 0.0
            assert abs(o.resid_mass[b].item() - p64[b].sum()) <= RTOL * p64[b].sum() + ATOL
        check_sampled_ids(p64[list(zero_rows)], us[list(zero_rows), 2], o.resid_ids.cpu().numpy()[list(zero_rows)],
                          np.array([oracle.sample_cdf(p64[b], us[b, 2]) for b in zero_rows]), what="token of a position without a draft")
    d, qd = rdk.rdk_sample_draft(ks, dev(q), 9, 0)
    assert all(d[b].item() == -1 and qd[b].item() == 0.0 for b in zero_rows)


# --------------------------------------------------------------------------------------------- fused entry point
@pytest.mark.parametrize("case", ["tiny", "ragged"])
@pytest.mark.parametrize("mode", ["sparse", "taylor"])
@pytest.mark.parametrize("kinds", [("prob", "prob"), ("logit", "logit")])
def test_fused_redistribute_verify(rdk, tiny, ragged, case, mode, kinds):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    p_kind, q_kind = kinds
    idx, wt, sw = data["sparse"]
    wt32, sw32 = wt.astype(np.float32), sw.astype(np.float32)
    if mode == "sparse":
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.SPARSE_TOPK, k=w.k, sparse=(dev(idx), dev(wt32), dev(sw32)))
        gmode = rdk.LINEAR_SPARSE
    else:
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.IDENTITY)
        gmode = rdk.LINEAR_TAYLOR
    p_in = dev(data["p"]) if p_kind == "prob" else dev(data["z_p"])
    q_in = dev(data["q_hat"]) if q_kind == "prob" else dev(data["z_q"])
    seed, offset = 4242, 17
    # with and without materialising q'
    qp_out = torch.zeros((w.B, w.N), dtype=torch.float32, device="cuda")
    o1 = rdk.rdk_redistribute_verify(kern, gmode, p_in, q_in, seed, offset, w.gamma, p_kind, q_kind, q_prime=qp_out)
    o2 = rdk.rdk_redistribute_verify(kern, gmode, p_in, q_in, seed, offset, w.gamma, p_kind, q_kind)
    torch.cuda.synchronize()
    two_call = rdk.rdk_redistribute_linear(kern, gmode, q_in, q_kind, p=p_in, p_kind=p_kind)
    assert torch.equal(qp_out, two_call)                    # the same kernel code produces q' in both entry points
    if mode == "sparse":      # the same block sums with and without the stores: identical outputs
        for name in ("draft_ids", "accept", "alpha", "resid_mass", "resid_ids", "n_accepted", "out_tokens"):
            assert torch.equal(getattr(o1, name), getattr(o2, name)), name
    # against the oracle chain
    p64 = data["p"].astype(np.float64) if p_kind == "prob" else oracle.probs_from(data["z_p"], "logit")
    ref_qp = oracle_rows(data, mode, q_kind, p_kind, kernel=(idx, wt32, sw32) if mode == "sparse" else None)
    assert_close(qp_out.cpu().numpy(), ref_qp, what="fused q'")
    ref = oracle.verify_batch(p64, ref_qp, seed, offset, gamma=w.gamma)
    check_verify_outputs(o2, ref, p64, ref_qp, seed, offset, w.gamma, p_kind)
    check_verify_outputs(o1, ref, p64, ref_qp, seed, offset, w.gamma, p_kind)   # Eq. 3 without q' sums its blocks another way
    # caller-supplied drafts through the fused path
    drafts = (np.arange(w.B, dtype=np.int32) * 11) % w.N
    o3 = rdk.rdk_redistribute_verify(kern, gmode, p_in, q_in, seed, offset, w.gamma, p_kind, q_kind, draft_ids=dev(drafts))
    ref3 = oracle.verify_batch(p64, ref_qp, seed, offset, sample_draft=False, draft_ids=drafts, gamma=w.gamma)
    check_verify_outputs(o3, ref3, p64, ref_qp, seed, offset, w.gamma, p_kind)


@pytest.mark.parametrize("shape", [(4102, 1021, 70, 7), (2049, 2049, 64, 8), (1500, 3, 96, 4), (9000, 4401, 130, 5)])
@pytest.mark.parametrize("kinds", [("prob", "prob"), ("prob", "logit"), ("logit", "logit"), ("logit", "prob"), ("bf16", "bf16")])
def test_fused_eq3_single_pass_ragged_shapes(rdk, shape, kinds):
    """The fused Eq. 3 call without q' takes one pass over the target rows once the batch has 64 positions (one workgroup
    per position, kept target values parked on chip; logit target rows from a vocabulary of 1024 ids on, with the softmax
    folded in: chunk maxima, power sums, one exp per id).  Shapes that end inside a chunk, inside a quad of slots and
    inside a 16-byte word; every id kept; three kept ids; more than half of the ids kept (slot runs longer than the
    registers hold); rows at a stride that rules the 16-byte paths out; probability, fp32-logit and bf16-logit rows on
    either side.  Against the oracle, and against the two-pass kernels."""
    N, n, B, gamma = shape
    p_kind, q_kind = kinds
    w = synth.scaled(synth.WORKLOADS["tiny"], name="rowshape", N=N, n=n, seqs=B // gamma, gamma=gamma, seed=N + n)
    data = make_inputs(w)
    kept = data["kept_ids"]
    kern = rdk.rdk_build_kernel(w.N, dev(kept), rdk.IDENTITY)
    z_p, z_q = data["z_p"], data["z_q"]
    if p_kind == "bf16":
        z_p, z_q = synth.bf16_round(z_p), synth.bf16_round(z_q)
    p64 = data["p"].astype(np.float64) if p_kind == "prob" else oracle.probs_from(z_p, "logit")
    q64 = data["q_hat"].astype(np.float64) if q_kind == "prob" else oracle.probs_from(z_q, "logit")
    p_src = data["p"] if p_kind == "prob" else z_p
    q_src = data["q_hat"] if q_kind == "prob" else z_q
    dt = torch.bfloat16 if p_kind == "bf16" else torch.float32
    pk = "prob" if p_kind == "prob" else "logit"
    qk = "prob" if q_kind == "prob" else "logit"
    ref_qp = oracle.redistribute_batch("taylor", q64, kept, w.N, p=p64)
    seed, offset = 515, 11
    ref = oracle.verify_batch(p64, ref_qp, seed, offset, gamma=gamma)
    for pad in (0, 3):                       # rows of a wider tensor: stride N + 3 keeps the rows off 16-byte boundaries
        p_big = torch.full((B, N + pad), float("nan"), dtype=dt, device="cuda")
        q_big = torch.full((B, n + pad), float("nan"), dtype=dt, device="cuda")
        p_big[:, :N] = dev(p_src).to(dt)
        q_big[:, :n] = dev(q_src).to(dt)
        o = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_TAYLOR, p_big[:, :N], q_big[:, :n], seed, offset, gamma, pk, qk)
        check_verify_outputs(o, ref, p64, ref_qp, seed, offset, gamma, pk, min_exact=0.9)
        qp = torch.empty((B, N), dtype=torch.float32, device="cuda")
        o2 = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_TAYLOR, p_big[:, :N], q_big[:, :n], seed, offset, gamma, pk, qk,
                                         q_prime=qp)
        assert_close(o.alpha.cpu().numpy(), o2.alpha.cpu().numpy(), what="alpha, one pass against two")
        assert_close(o.resid_mass.cpu().numpy(), o2.resid_mass.cpu().numpy(), what="residual mass, one pass against two")
        assert (o.draft_ids == o2.draft_ids).float().mean().item() >= 0.95
    # caller-supplied drafts through the same kernel (their two values are fetched in the finish)
    drafts = (np.arange(B, dtype=np.int32) * 11) % N
    o3 = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_TAYLOR, p_big[:, :N], q_big[:, :n], seed, offset, gamma, pk, qk,
                                     draft_ids=dev(drafts))
    ref3 = oracle.verify_batch(p64, ref_qp, seed, offset, sample_draft=False, draft_ids=drafts, gamma=gamma)
    check_verify_outputs(o3, ref3, p64, ref_qp, seed, offset, gamma, pk, min_exact=0.9)


def test_fused_eq3_single_pass_many_chunks(rdk):
    """A vocabulary of 391 chunks with a few dozen kept ids in each: more pieces of kept slots (one per chunk and one per
    64 slots, here about 700) than the groups of the one-pass kernel are handed before the row constants are known, so the
    rest is fetched in the second step itself."""
    w = synth.scaled(synth.WORKLOADS["tiny"], name="manychunks", N=400003, n=20011, seqs=8, gamma=8, seed=31)
    data = make_inputs(w)
    kept = data["kept_ids"]
    assert np.unique(kept // 1024).size + kept.size // 64 > 640
    kern = rdk.rdk_build_kernel(w.N, dev(kept), rdk.IDENTITY)
    p64, q64 = data["p"].astype(np.float64), data["q_hat"].astype(np.float64)
    ref_qp = oracle.redistribute_batch("taylor", q64, kept, w.N, p=p64)
    seed, offset = 808, 3
    ref = oracle.verify_batch(p64, ref_qp, seed, offset, gamma=w.gamma)
    o = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_TAYLOR, dev(data["p"]), dev(data["q_hat"]), seed, offset, w.gamma)
    check_verify_outputs(o, ref, p64, ref_qp, seed, offset, w.gamma, "prob", min_exact=0.9)


def test_large_batch_with_more_block_sums_than_registers(rdk):
    """586 block sums of 1024 ids per row (N > 2^19) in a batch of 128 positions: the finish that eight wavefronts share
    then re-reads the block sums when it locates the crossings instead of keeping them in registers -- out of LDS in the
    one-pass Eq. 3 kernel, out of memory in the stand-alone verification and in the two-pass Eq. 3 path."""
    w = synth.scaled(synth.WORKLOADS["tiny"], name="wide128", N=600011, n=3001, seqs=16, gamma=8, seed=37)
    data = make_inputs(w)
    kept = data["kept_ids"]
    kern = rdk.rdk_build_kernel(w.N, dev(kept), rdk.IDENTITY)
    p64, q64 = data["p"].astype(np.float64), data["q_hat"].astype(np.float64)
    ref_qp = oracle.redistribute_batch("taylor", q64, kept, w.N, p=p64)
    seed, offset = 909, 6
    ref = oracle.verify_batch(p64, ref_qp, seed, offset, gamma=w.gamma)
    p_d, q_d = dev(data["p"]), dev(data["q_hat"])
    rdk.rdk_timing_select("taylor_row_kernel")
    o = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_TAYLOR, p_d, q_d, seed, offset, w.gamma)
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    assert rdk.rdk_timing_read("taylor_row_kernel")[0] == 1          # the one-pass kernel took this call
    check_verify_outputs(o, ref, p64, ref_qp, seed, offset, w.gamma, "prob", min_exact=0.9)
    rows = torch.empty(w.B, w.N, device="cuda")
    o2 = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_TAYLOR, p_d, q_d, seed, offset, w.gamma, q_prime=rows)
    check_verify_outputs(o2, ref, p64, ref_qp, seed, offset, w.gamma, "prob", min_exact=0.9)
    qp32 = rows.cpu().numpy()
    assert_close(qp32, ref_qp, what="q' of the fused call")
    run_verify_case(rdk, p_d, "prob", p64, qp32, w.gamma, seed=910, offset=0)
    drafts = (np.arange(w.B, dtype=np.int32) * 50021) % w.N
    run_verify_case(rdk, p_d, "prob", p64, qp32, w.gamma, seed=911, offset=1, draft_ids=drafts)


# --------------------------------------------------------------------------------------------- HIP graph capture
@pytest.mark.parametrize("mode", ["sparse", "taylor"])
def test_fused_call_replays_from_a_hip_graph(rdk, ragged, mode):
    """The fused call only enqueues kernels on the caller's stream (no allocation, no memset, no synchronisation),
    so a serving loop can capture it once and replay it.  Three replays on three different batches, with eager work
    and synchronisations between them, each compared with the eager call on the same inputs."""
    data = ragged
    w = data["w"]
    idx, wt, sw = data["sparse"]
    if mode == "sparse":
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.SPARSE_TOPK, k=w.k,
                                    sparse=(dev(idx), dev(wt.astype(np.float32)), dev(sw.astype(np.float32))))
        gmode = rdk.LINEAR_SPARSE
    else:
        kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.IDENTITY)
        gmode = rdk.LINEAR_TAYLOR
    seed, offset = 99, 5
    p_static, q_static = dev(data["p"]).clone(), dev(data["q_hat"]).clone()
    captured = rdk.VerifyOutputs(w.B, w.N, w.gamma, p_static.device)
    eager = rdk.VerifyOutputs(w.B, w.N, w.gamma, p_static.device)
    # one eager call first: sizes the workspaces outside the capture
    rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=captured)
    rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=eager)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=captured)
    rng = np.random.default_rng(5)
    for rep in range(3):
        perm = rng.permutation(w.B)
        p_static.copy_(dev(data["p"][perm]))
        q_static.copy_(dev(data["q_hat"][perm]))
        for name in ("draft_ids", "resid_ids"):
            getattr(captured, name).fill_(-7)
        captured.alpha.zero_()
        graph.replay()
        torch.cuda.synchronize()
        rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=eager)
        torch.cuda.synchronize()
        for name in ("draft_ids", "accept", "alpha", "resid_mass", "resid_ids", "n_accepted", "out_tokens"):
            assert torch.equal(getattr(captured, name), getattr(eager, name)), "replay %d: %s" % (rep, name)


@pytest.mark.parametrize("mode", ["sparse", "taylor"])
def test_fused_call_of_a_large_batch_replays_from_a_hip_graph(rdk, mode):
    """256 positions: the batch shape at which Eq. 3 takes its one-pass kernel (finish inside) and the sparse form finishes
    every row on a workgroup of its own, rows dealt out by XCD, with the per-sequence scan as a launch of its own.  The
    captured call against the oracle once, then three replays on permuted batches against the eager call."""
    w = synth.scaled(synth.WORKLOADS["tiny"], name="graphbatch", N=4102, n=1021, k=16, seqs=32, gamma=8, seed=77)
    data = make_inputs(w)
    kept = data["kept_ids"]
    if mode == "sparse":
        idx, wt, sw = stochastic_topk_kernel(np.random.default_rng(3), w.N, kept, w.k)
        kern = rdk.rdk_build_kernel(w.N, dev(kept), rdk.SPARSE_TOPK, k=w.k,
                                    sparse=(dev(idx), dev(wt.astype(np.float32)), dev(sw.astype(np.float32))))
        gmode = rdk.LINEAR_SPARSE
        sparse32 = (idx, wt.astype(np.float32).astype(np.float64), sw.astype(np.float32).astype(np.float64))
        ref_qp = oracle.redistribute_batch("sparse", data["q_hat"].astype(np.float64), kept, w.N, sparse=sparse32)
    else:
        kern = rdk.rdk_build_kernel(w.N, dev(kept), rdk.IDENTITY)
        gmode = rdk.LINEAR_TAYLOR
        ref_qp = oracle.redistribute_batch("taylor", data["q_hat"].astype(np.float64), kept, w.N, p=data["p"].astype(np.float64))
    seed, offset = 4242, 9
    p_static, q_static = dev(data["p"]).clone(), dev(data["q_hat"]).clone()
    captured = rdk.VerifyOutputs(w.B, w.N, w.gamma, p_static.device)
    eager = rdk.VerifyOutputs(w.B, w.N, w.gamma, p_static.device)
    rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=captured)
    rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=eager)
    torch.cuda.synchronize()
    p64 = data["p"].astype(np.float64)
    check_verify_outputs(eager, oracle.verify_batch(p64, ref_qp, seed, offset, gamma=w.gamma), p64, ref_qp, seed, offset, w.gamma,
                         "prob", min_exact=0.9)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=captured)
    rng = np.random.default_rng(6)
    for rep in range(3):
        perm = rng.permutation(w.B)
        p_static.copy_(dev(data["p"][perm]))
        q_static.copy_(dev(data["q_hat"][perm]))
        for name in ("draft_ids", "resid_ids"):
            getattr(captured, name).fill_(-7)
        captured.alpha.zero_()
        graph.replay()
        torch.cuda.synchronize()
        rdk.rdk_redistribute_verify(kern, gmode, p_static, q_static, seed, offset, w.gamma, outputs=eager)
        torch.cuda.synchronize()
        for name in ("draft_ids", "accept", "alpha", "resid_mass", "resid_ids", "n_accepted", "out_tokens"):
            assert torch.equal(getattr(captured, name), getattr(eager, name)), "replay %d: %s" % (rep, name)


def test_kernel_timing_brackets_every_nth_launch(rdk, ragged):
    """rdk_timing_select("name/4"): of the launches of that kernel every fourth is bracketed by events."""
    data = ragged
    w = data["w"]
    p, q = dev(data["p"]), dev(data["p"][::-1].copy())              # any q' rows will do
    out = rdk.VerifyOutputs(w.B, w.N, w.gamma, p.device)
    rdk.rdk_timing_select("verify_stream_kernel/4")
    for i in range(8):
        rdk.rdk_verify_sample(p, q, seed=1, offset=i, gamma=w.gamma, outputs=out)
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    count, ms = rdk.rdk_timing_read("verify_stream_kernel")
    assert count == 2 and ms > 0.0
    rdk.rdk_timing_select("verify_stream_kernel")
    for i in range(3):
        rdk.rdk_verify_sample(p, q, seed=1, offset=i, gamma=w.gamma, outputs=out)
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    assert rdk.rdk_timing_read("verify_stream_kernel")[0] == 3
    assert rdk.rdk_timing_read("verify_stream_kernel")[0] == 0    # read forgets


# --------------------------------------------------------------------------------------------- degenerate shapes
DEGENERATE = {
    "one_row": dict(N=40, n=7, k=3, seqs=1, gamma=1, d=8),                # a single position, a vocabulary below one tile
    "nothing_pruned": dict(N=300, n=300, k=4, seqs=2, gamma=2, d=8),      # n = N: the kernel is the identity
    "one_kept": dict(N=129, n=1, k=1, seqs=1, gamma=3, d=8),              # the drafter knows a single token
    "no_neighbours": dict(N=1000, n=100, k=0, seqs=5, gamma=1, d=8),      # top-0: the sparse form is TLI
}


@pytest.mark.parametrize("shape", sorted(DEGENERATE))
def test_degenerate_shapes(rdk, shape):
    """The smallest and the limiting shapes the method allows, through every redistribution form and the fused call."""
    w = synth.scaled(synth.WORKLOADS["tiny"], name=shape, seed=7, **DEGENERATE[shape])
    data = make_inputs(w)
    data["w"] = w
    kept = dev(data["kept_ids"])
    idx, wt, sw = oracle.build_sparse(data["E"], data["kept_ids"], w.tau, w.k)
    wt32, sw32 = wt.astype(np.float32), sw.astype(np.float32)
    M32 = oracle.build_dense(data["E"], data["kept_ids"], w.tau).astype(np.float32)
    p64 = data["p"].astype(np.float64)
    q, p = dev(data["q_hat"]), dev(data["p"])

    ks = rdk.rdk_build_kernel(w.N, kept, rdk.SPARSE_TOPK, k=w.k, sparse=(dev(idx), dev(wt32), dev(sw32)))
    ref_sparse = oracle.redistribute_batch("sparse", data["q_hat"], data["kept_ids"], w.N, sparse=(idx, wt32, sw32))
    assert_close(rdk.rdk_redistribute_linear(ks, rdk.LINEAR_SPARSE, q).cpu().numpy(), ref_sparse, what="sparse q'")
    if w.k > 0 and w.n < w.N:   # the device-built kernel of the same shape
        kb = rdk.rdk_build_kernel(w.N, kept, rdk.SPARSE_TOPK, embeddings=dev(data["E"]), tau=w.tau, k=w.k)
        b_idx, b_w, b_sw = [t.cpu().numpy() for t in rdk.rdk_kernel_get_sparse(kb)]
        assert np.array_equal(b_idx, idx)
        assert_close(b_w, wt, what="neighbour weights")
        assert_close(b_sw, sw, what="diagonal weights")
    if w.k == 0 or w.n == w.N:   # nothing but the diagonal: token-level intersection
        ref_tli = oracle.redistribute_batch("exact", data["q_hat"], data["kept_ids"], w.N,
                                            M=np.eye(w.N)[data["kept_ids"]])
        assert_close(ref_sparse, ref_tli, what="oracle: sparse form without neighbours is TLI")

    ki = rdk.rdk_build_kernel(w.N, kept, rdk.IDENTITY)
    ref_taylor = oracle.redistribute_batch("taylor", data["q_hat"], data["kept_ids"], w.N, p=data["p"])
    assert_close(rdk.rdk_redistribute_linear(ki, rdk.LINEAR_TAYLOR, q, p=p).cpu().numpy(), ref_taylor, what="Eq. 3 q'")
    # logit inputs at a vocabulary too small for the one-pass statistics: the softmax pass followed by the two-pass sums
    ref_logit = oracle.redistribute_batch("taylor", oracle.probs_from(data["z_q"], "logit"), data["kept_ids"], w.N,
                                          p=oracle.probs_from(data["z_p"], "logit"))
    got = rdk.rdk_redistribute_linear(ki, rdk.LINEAR_TAYLOR, dev(data["z_q"]), "logit", p=dev(data["z_p"]), p_kind="logit")
    assert_close(got.cpu().numpy(), ref_logit, what="Eq. 3 q' from logits")

    ref_exact = oracle.redistribute_batch("exact", data["q_hat"], data["kept_ids"], w.N, M=M32)
    kd = rdk.rdk_build_kernel(w.N, kept, rdk.DENSE_F32, dense_M=dev(M32))
    assert_close(rdk.rdk_redistribute_exact(kd, q).cpu().numpy(), ref_exact, what="exact fp32")
    kh = rdk.rdk_build_kernel(w.N, kept, rdk.DENSE_BF16, dense_M=dev(M32))
    ref_stored = oracle.redistribute_batch("exact", data["q_hat"], data["kept_ids"], w.N, M=operand_round_M(M32))
    ref_stored /= ref_stored.sum(1, keepdims=True)
    got_h = rdk.rdk_redistribute_exact(kh, q).cpu().numpy()
    assert_close(got_h, ref_stored, rtol=RTOL_DENSE, atol=ATOL, what="exact bf16 vs the stored kernel")
    assert_close(got_h, ref_exact, rtol=RTOL_DENSE_UNROUNDED, atol=ATOL, what="exact bf16 vs fp32 kernel")

    seed, offset = 31, 2
    for kern, gmode, ref_qp in ((ks, rdk.LINEAR_SPARSE, ref_sparse), (ki, rdk.LINEAR_TAYLOR, ref_taylor)):
        o = rdk.rdk_redistribute_verify(kern, gmode, p, q, seed, offset, w.gamma)
        ref = oracle.verify_batch(p64, ref_qp, seed, offset, gamma=w.gamma)
        check_verify_outputs(o, ref, p64, ref_qp, seed, offset, w.gamma, "prob", min_exact=0.0)   # ids: near-ties only
    qp32 = ref_sparse.astype(np.float32)
    o = rdk.rdk_verify_sample(p, dev(qp32), seed, offset, w.gamma)
    ref = oracle.verify_batch(p64, qp32.astype(np.float64), seed, offset, gamma=w.gamma)
    check_verify_outputs(o, ref, p64, qp32.astype(np.float64), seed, offset, w.gamma, "prob", min_exact=0.0)
    ids, _ = rdk.rdk_sample_draft(ks, q, seed, offset)
    u0 = np.array([oracle.uniforms(seed, offset + b)[0] for b in range(w.B)])
    ref_ids = np.array([oracle.sample_cdf(ref_sparse[b], u0[b]) for b in range(w.B)])
    check_sampled_ids(ref_sparse, u0, ids.cpu().numpy(), ref_ids, what="draft from q'")


# --------------------------------------------------------------------------------------------- concurrent streams
def test_calls_on_two_streams_with_their_own_workspaces(rdk, ragged):
    """Two fused calls that share the kernel handle but not their workspaces, enqueued on two streams so that they
    overlap, give what each gives alone."""
    data = ragged
    w = data["w"]
    idx, wt, sw = data["sparse"]
    ks = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.SPARSE_TOPK, k=w.k,
                              sparse=(dev(idx), dev(wt.astype(np.float32)), dev(sw.astype(np.float32))))
    ki = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.IDENTITY)
    p, q = dev(data["p"]), dev(data["q_hat"])
    p2, q2 = dev(data["p"][::-1].copy()), dev(data["q_hat"][::-1].copy())
    alone = [rdk.rdk_redistribute_verify(ks, rdk.LINEAR_SPARSE, p, q, 5, 0, w.gamma),
             rdk.rdk_redistribute_verify(ki, rdk.LINEAR_TAYLOR, p2, q2, 6, 100, w.gamma)]
    torch.cuda.synchronize()
    outs = [rdk.VerifyOutputs(w.B, w.N, w.gamma, p.device) for _ in range(2)]
    for o in outs:   # sizes the fused workspaces before the streams start
        rdk.rdk_redistribute_verify(ks, rdk.LINEAR_SPARSE, p, q, 5, 0, w.gamma, outputs=o)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(10):
        with torch.cuda.stream(streams[0]):
            rdk.rdk_redistribute_verify(ks, rdk.LINEAR_SPARSE, p, q, 5, 0, w.gamma, outputs=outs[0])
        with torch.cuda.stream(streams[1]):
            rdk.rdk_redistribute_verify(ki, rdk.LINEAR_TAYLOR, p2, q2, 6, 100, w.gamma, outputs=outs[1])
    torch.cuda.synchronize()
    for got, ref in zip(outs, alone):
        for name in ("draft_ids", "accept", "alpha", "resid_mass", "resid_ids", "n_accepted", "out_tokens"):
            assert torch.equal(getattr(got, name), getattr(ref, name)), name


# --------------------------------------------------------------------------------------------- long neighbour rows
@pytest.mark.parametrize("k", [17, 32, 40])
def test_sparse_rows_longer_than_one_round(rdk, ragged, k):
    """More than sixteen neighbours per pruned id: the product runs several rounds per id and the finish kernel
    re-computes its two blocks round by round.  Fused call against the oracle, its q' bit-equal to the two-call rows,
    and the draft draw bit-equal to the fused call's."""
    data = ragged
    w = data["w"]
    idx, wt, sw = stochastic_topk_kernel(np.random.default_rng(40 + k), w.N, data["kept_ids"], k)
    wt, sw = wt.astype(np.float32), sw.astype(np.float32)          # the kernel as both sides store it
    kern = rdk.rdk_build_kernel(w.N, dev(data["kept_ids"]), rdk.SPARSE_TOPK, k=k, sparse=(dev(idx), dev(wt), dev(sw)))
    p, q = dev(data["p"]), dev(data["q_hat"])
    seed, offset = 77, 9
    qp = torch.zeros((w.B, w.N), dtype=torch.float32, device="cuda")
    o = rdk.rdk_redistribute_verify(kern, rdk.LINEAR_SPARSE, p, q, seed, offset, w.gamma, q_prime=qp)
    rows = rdk.rdk_redistribute_linear(kern, rdk.LINEAR_SPARSE, q)
    assert torch.equal(qp, rows)
    ref_qp = oracle.redistribute_batch("sparse", data["q_hat"], data["kept_ids"], w.N, sparse=(idx, wt, sw))
    assert_close(qp.cpu().numpy(), ref_qp, what="sparse q', k=%d" % k)
    p64 = data["p"].astype(np.float64)
    ref = oracle.verify_batch(p64, ref_qp, seed, offset, gamma=w.gamma)
    check_verify_outputs(o, ref, p64, ref_qp, seed, offset, w.gamma, "prob")
    ids, qd = rdk.rdk_sample_draft(kern, q, seed, offset)
    assert torch.equal(ids, o.draft_ids)
    assert_close(qd.cpu().numpy(), ref_qp[np.arange(w.B), ids.cpu().numpy()], what="q' at the drafted id")


# --------------------------------------------------------------------------------------------- padded rows, random shapes
def padded(a, pad, dtype=None, fill=float("nan")):
    """Device view [B, width] of a wider tensor whose extra columns hold `fill`: a row stride above the width."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    big = torch.full((t.shape[0], t.shape[1] + pad), fill, dtype=t.dtype)
    big[:, :t.shape[1]] = t
    big = big.cuda()
    return big[:, :t.shape[1]], big


def draw_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    edges = [63, 64, 65, 255, 257, 511, 512, 513, 1023, 1024, 1025, 1535, 2047, 2049, 4095, 4097]
    N = int(rng.choice(edges)) if rng.random() < 0.6 else int(rng.integers(5, 5000))
    n = int(rng.integers(1, N + 1)) if rng.random() < 0.8 else int(rng.choice([1, max(1, N // 2), N]))
    k = min(n, int(rng.choice([0, 1, 3, 8, 15, 16, 17, 33])))
    # row strides: the width itself, the next multiple of four (the 16-byte paths with a ragged end), and wider
    pads = [int(rng.choice([0, (-w_) % 4, (-w_) % 4 + 4, 1, 3])) for w_ in (N, n, N)]
    return dict(N=N, n=n, k=k, seqs=int(rng.integers(1, 7)), gamma=int(rng.integers(1, 5)), d=int(rng.integers(4, 33))), pads, rng


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_with_padded_rows(rdk, seed):
    """Shapes drawn around the tile, block and vector-width boundaries, inputs and outputs as views of wider
    tensors (row stride above the width, padding poisoned): nothing past a row's width may be read or written."""
    shape, (pad_p, pad_q, pad_o), rng = draw_shape(seed)
    w = synth.scaled(synth.WORKLOADS["tiny"], name="random%d" % seed, seed=100 + seed, **shape)
    data = make_inputs(w)
    data["w"] = w
    kinds = ("prob", "logit", "bf16")[seed % 3]
    if kinds == "bf16":
        data["z_p"], data["z_q"] = synth.bf16_round(data["z_p"]), synth.bf16_round(data["z_q"])
    print("seed", seed, shape, "pads", (pad_p, pad_q, pad_o), kinds, flush=True)
    kept = dev(data["kept_ids"])
    if 0 < w.k <= w.n // 2:
        idx, wt, sw = stochastic_topk_kernel(rng, w.N, data["kept_ids"], w.k)
    else:   # no neighbours, or most of the kept slots: the top-k kernel of the embeddings (distinct by construction)
        idx, wt, sw = oracle.build_sparse(data["E"], data["kept_ids"], w.tau, w.k)
    wt32, sw32 = np.asarray(wt, np.float32), np.asarray(sw, np.float32)
    if kinds == "prob":
        p_in, p_big = padded(data["p"], pad_p)
        q_in, q_big = padded(data["q_hat"], pad_q)
        pk = qk = "prob"
        p64, q64 = data["p"].astype(np.float64), data["q_hat"].astype(np.float64)
    else:
        dt = torch.bfloat16 if kinds == "bf16" else None
        p_in, p_big = padded(data["z_p"], pad_p, dt)
        q_in, q_big = padded(data["z_q"], pad_q, dt)
        pk = qk = "logit"
        p64, q64 = oracle.probs_from(data["z_p"], "logit"), oracle.probs_from(data["z_q"], "logit")
    sentinel = -123.0

    def out_view():
        big = torch.full((w.B, w.N + pad_o), sentinel, dtype=torch.float32, device="cuda")
        return big[:, :w.N], big

    def check_rows(view, big, ref, what):
        assert_close(view.cpu().numpy(), ref, what=what)
        assert bool((big[:, w.N:] == sentinel).all()), what + ": wrote past the row"

    ks = rdk.rdk_build_kernel(w.N, kept, rdk.SPARSE_TOPK, k=w.k, sparse=(dev(idx), dev(wt32), dev(sw32)))
    ki = rdk.rdk_build_kernel(w.N, kept, rdk.IDENTITY)
    ref_sparse = oracle.redistribute_batch("sparse", q64, data["kept_ids"], w.N, sparse=(idx, wt32, sw32))
    ref_taylor = oracle.redistribute_batch("taylor", q64, data["kept_ids"], w.N, p=p64)
    seed_, offset = 77 + seed, 5
    for kern, gmode, ref_qp, name in ((ks, rdk.LINEAR_SPARSE, ref_sparse, "sparse"), (ki, rdk.LINEAR_TAYLOR, ref_taylor, "Eq. 3")):
        view, big = out_view()
        rdk.rdk_redistribute_linear(kern, gmode, q_in, qk, p=p_in, p_kind=pk, out=view)
        check_rows(view, big, ref_qp, name + " q'")
        ref = oracle.verify_batch(p64, ref_qp, seed_, offset, gamma=w.gamma)
        view2, big2 = out_view()
        o1 = rdk.rdk_redistribute_verify(kern, gmode, p_in, q_in, seed_, offset, w.gamma, pk, qk, q_prime=view2)
        check_rows(view2, big2, ref_qp, name + " fused q'")
        assert torch.equal(view, view2)
        o2 = rdk.rdk_redistribute_verify(kern, gmode, p_in, q_in, seed_, offset, w.gamma, pk, qk)
        for o in (o1, o2):
            check_verify_outputs(o, ref, p64, ref_qp, seed_, offset, w.gamma, pk, min_exact=0.0)
        # the materialised rows (padded) through the stand-alone verification
        qp32 = view.cpu().numpy()
        o3 = rdk.rdk_verify_sample(p_in, view, seed_, offset, w.gamma, pk)
        ref3 = oracle.verify_batch(p64, qp32.astype(np.float64), seed_, offset, gamma=w.gamma)
        check_verify_outputs(o3, ref3, p64, qp32.astype(np.float64), seed_, offset, w.gamma, pk, min_exact=0.0)
    # several candidates per position on the materialised (padded) rows of the sparse form
    view, big = out_view()
    rdk.rdk_redistribute_linear(ks, rdk.LINEAR_SPARSE, q_in, qk, out=view)
    C = 1 + seed % 4
    qp64 = view.cpu().numpy().astype(np.float64)
    refm = oracle.verify_multi_batch(p64, qp64, C, seed_, offset)
    om = rdk.rdk_verify_multi(p_in, view, C, seed_, offset, pk, cand_ids=dev(refm["cand_ids"]))
    check_multi(om, refm, p64, qp64, seed_, offset, C, min_exact=0.0)
    # draft draw before any target row exists
    view, big = out_view()
    ids, _ = rdk.rdk_sample_draft(ks, q_in, seed_, offset, qk, q_prime=view)
    check_rows(view, big, ref_sparse, "draft q'")
    u0 = np.array([oracle.uniforms(seed_, offset + b)[0] for b in range(w.B)])
    ref_ids = np.array([oracle.sample_cdf(ref_sparse[b], u0[b]) for b in range(w.B)])
    check_sampled_ids(ref_sparse, u0, ids.cpu().numpy(), ref_ids, what="draft from q'")
    # exact forms on a random row-stochastic kernel
    if w.n * w.N <= 4_000_000:
        M32 = random_row_stochastic(rng, w.n, w.N).astype(np.float32)
        ref_exact = oracle.redistribute_batch("exact", q64, data["kept_ids"], w.N, M=M32)
        for fmt, tol in ((rdk.DENSE_F32, dict()), (rdk.DENSE_BF16, dict(rtol=RTOL_DENSE_UNROUNDED, atol=ATOL))):
            kd = rdk.rdk_build_kernel(w.N, kept, fmt, dense_M=dev(M32))
            view, big = out_view()
            rdk.rdk_redistribute_exact(kd, q_in, qk, out=view)
            assert_close(view.cpu().numpy(), ref_exact, what="exact", **tol)
            assert bool((big[:, w.N:] == sentinel).all()), "exact: wrote past the row"
    # the inputs are untouched, padding included
    assert bool(torch.isnan(p_big[:, w.N:].float()).all()) and bool(torch.isnan(q_big[:, w.n:].float()).all())


# --------------------------------------------------------------------------------------------- several candidates per position
@pytest.mark.parametrize("case", ["tiny", "ragged"])
@pytest.mark.parametrize("p_kind", ["prob", "logit"])
@pytest.mark.parametrize("C", [1, 3, 6])
def test_verify_multi(rdk, tiny, ragged, case, p_kind, C):
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    idx, wt, sw = data["sparse"]
    qp32 = oracle_rows(data, "sparse", kernel=(idx, wt.astype(np.float32), sw.astype(np.float32))).astype(np.float32)
    q64 = qp32.astype(np.float64)
    p64 = data["p"].astype(np.float64) if p_kind == "prob" else oracle.probs_from(data["z_p"], "logit")
    p_in = dev(data["p"]) if p_kind == "prob" else dev(data["z_p"])
    seed, offset = 900 + C, (1 << 33) + 5
    ref = oracle.verify_multi_batch(p64, q64, C, seed, offset)
    # candidates drawn by the library: each is the inverse-CDF draw of q' under its own uniform
    o = rdk.rdk_verify_multi(p_in, dev(qp32), C, seed, offset, p_kind)
    g_cand = o.cand_ids.cpu().numpy()
    for i in range(C):
        us = np.array([oracle.multi_uniform(seed, offset + b, i) for b in range(w.B)])
        check_sampled_ids(q64, us, g_cand[:, i], ref["cand_ids"][:, i], what="candidate %d" % i)
    if np.array_equal(g_cand, ref["cand_ids"]):
        check_multi(o, ref, p64, q64, seed, offset, C)
    # the oracle's candidates handed to the library: the rounds alone
    o2 = rdk.rdk_verify_multi(p_in, dev(qp32), C, seed, offset, p_kind, cand_ids=dev(ref["cand_ids"]))
    assert np.array_equal(o2.cand_ids.cpu().numpy(), ref["cand_ids"])
    check_multi(o2, ref, p64, q64, seed, offset, C)
    # candidates that can never be kept (outside the vocabulary, or without drafter mass): all rounds, then the residual
    bad = np.full((w.B, C), -1, np.int32)
    bad[:, ::2] = w.N + 7
    ref3 = oracle.verify_multi_batch(p64, q64, C, seed, offset, cand_ids=bad)
    o3 = rdk.rdk_verify_multi(p_in, dev(qp32), C, seed, offset, p_kind, cand_ids=dev(bad))
    assert (o3.accepted.cpu().numpy() == C).all() and (ref3["accepted"] == C).all()
    check_multi(o3, ref3, p64, q64, seed, offset, C, min_exact=0.8)


def test_verify_multi_with_one_candidate_is_verify_sample(rdk, ragged):
    """C = 1 through the new entry point and Alg. 4 through rdk_verify_sample: same draft, decision and token."""
    w = ragged["w"]
    idx, wt, sw = ragged["sparse"]
    qp32 = oracle_rows(ragged, "sparse", kernel=(idx, wt.astype(np.float32), sw.astype(np.float32))).astype(np.float32)
    p, qp = dev(ragged["p"]), dev(qp32)
    one = rdk.rdk_verify_sample(p, qp, 55, 9, 0)
    multi = rdk.rdk_verify_multi(p, qp, 1, 55, 9)
    torch.cuda.synchronize()
    assert torch.equal(multi.cand_ids[:, 0], one.draft_ids)
    assert torch.equal(multi.accepted == 0, one.accept == 1)
    assert torch.equal(multi.token, torch.where(one.accept == 1, one.draft_ids, one.resid_ids))


def test_verify_multi_edges_and_errors(rdk, tiny):
    w = tiny["w"]
    p = dev(tiny["p"])
    # p = q': the first candidate is always kept
    o = rdk.rdk_verify_multi(p, p, 4, 3, 0)
    assert not o.accepted.any() and torch.equal(o.token, o.cand_ids[:, 0]) and not o.resid_mass.any()
    # a drafter row without mass: no candidate (-1), the token is drawn from p itself (first residual = p)
    zero = torch.zeros_like(p)
    o = rdk.rdk_verify_multi(p, zero, 2, 3, 0)
    ref = oracle.verify_multi_batch(tiny["p"].astype(np.float64), np.zeros((w.B, w.N)), 2, 3, 0)
    assert (o.cand_ids.cpu().numpy() == -1).all() and (ref["cand_ids"] == -1).all()
    assert (o.accepted.cpu().numpy() == 2).all()
    check_multi(o, ref, tiny["p"].astype(np.float64), np.zeros((w.B, w.N)), 3, 0, 2)
    for kwargs, status in ((dict(C=0), 2), (dict(C=17), 7)):
        with pytest.raises(rdk.RdkError) as e:
            rdk.rdk_verify_multi(p, p, kwargs["C"], 1, 0)
        assert e.value.status == status


@pytest.mark.parametrize("case", ["tiny", "ragged"])
def test_tree_verification(rdk, tiny, ragged, case):
    """Token trees: every node verified with its children as candidates (lists of 0 .. C ids), then the walk."""
    data = tiny if case == "tiny" else ragged
    w = data["w"]
    nodes, C = (4, 2) if case == "tiny" else (7, 3)
    S = w.B // nodes
    B = S * nodes
    idx, wt, sw = data["sparse"]
    qp32 = oracle_rows(data, "sparse", kernel=(idx, wt.astype(np.float32), sw.astype(np.float32))).astype(np.float32)[:B]
    q64, p64 = qp32.astype(np.float64), data["p"].astype(np.float64)[:B]
    seed, offset = 321, 77
    child, cand = random_trees(np.random.default_rng(8), S, nodes, C, q64, seed, offset)
    assert (cand[:, 0] < 0).any() and (cand[:, -1] >= 0).any()          # leaves and full nodes both occur
    ref = oracle.verify_multi_batch(p64, q64, C, seed, offset, cand_ids=cand)
    ref_n, ref_tok = oracle.tree_walk(child, ref["accepted"], ref["token"], S, nodes, C)
    o = rdk.rdk_verify_multi(dev(data["p"][:B]), dev(qp32), C, seed, offset, cand_ids=dev(cand))
    check_multi(o, ref, p64, q64, seed, offset, C, min_exact=0.85)
    # the walk is integer work: on the oracle's per-node results it must give the oracle's paths bit for bit
    n_acc, toks = rdk.rdk_tree_walk(dev(child), dev(ref["accepted"]), dev(ref["token"]))
    assert np.array_equal(n_acc.cpu().numpy(), ref_n) and np.array_equal(toks.cpu().numpy(), ref_tok)
    # and on the device's own results, the oracle's walk of those results
    n_acc, toks = rdk.rdk_tree_walk(dev(child), o.accepted, o.token)
    own_n, own_tok = oracle.tree_walk(child, o.accepted.cpu().numpy(), o.token.cpu().numpy(), S, nodes, C)
    assert np.array_equal(n_acc.cpu().numpy(), own_n) and np.array_equal(toks.cpu().numpy(), own_tok)
    same = (o.accepted.cpu().numpy() == ref["accepted"]) & (o.token.cpu().numpy() == ref["token"])
    if same.all():
        assert np.array_equal(toks.cpu().numpy(), ref_tok)
    # a walk that does not describe a tree stops instead of looping
    loop = child.copy()
    loop[:, :, :] = 0
    n_acc, toks = rdk.rdk_tree_walk(dev(loop), dev(np.zeros(B, np.int32)), dev(ref["token"]))
    assert not n_acc.any() and np.array_equal(toks.cpu().numpy()[:, 0], ref["token"][::nodes])
    with pytest.raises(rdk.RdkError):
        rdk.rdk_tree_walk(dev(child[:, :, :0].copy()), o.accepted, o.token)


def test_tree_verification_replays_from_a_hip_graph(rdk, ragged):
    """rdk_verify_multi + rdk_tree_walk recorded once and replayed on fresh inputs: every replay equals the eager calls."""
    w = ragged["w"]
    nodes, C = 7, 3
    S = w.B // nodes
    B = S * nodes
    idx, wt, sw = ragged["sparse"]
    qp32 = oracle_rows(ragged, "sparse", kernel=(idx, wt.astype(np.float32), sw.astype(np.float32))).astype(np.float32)[:B]
    child, cand = random_trees(np.random.default_rng(8), S, nodes, C, qp32.astype(np.float64), 5, 0)
    p_static, q_static, cand_d, child_d = dev(ragged["p"][:B]).clone(), dev(qp32).clone(), dev(cand), dev(child)
    captured, eager = rdk.MultiOutputs(B, C, p_static.device), rdk.MultiOutputs(B, C, p_static.device)
    n_cap = torch.zeros(S, dtype=torch.int32, device="cuda")
    t_cap = torch.zeros((S, nodes), dtype=torch.int32, device="cuda")

    def call(o, n_out=None, t_out=None):
        o.cand_ids.copy_(cand_d)
        d = rdk.MultiDesc(B=B, N=w.N, C=C, seed=5, offset=0, sample_candidates=0)
        L = rdk.lib()
        st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        P = lambda t: ctypes.c_void_p(t.data_ptr())
        assert L.rdk_verify_multi(ctypes.byref(d), P(p_static), 0, w.N, P(q_static), w.N, P(o.cand_ids), P(o.accepted), P(o.token),
                                  P(o.resid_mass), P(o.ws), o.ws.numel(), st) == 0
        if n_out is not None:
            assert L.rdk_tree_walk(S, nodes, C, P(child_d), P(o.accepted), P(o.token), P(n_out), P(t_out), st) == 0

    for o in (captured, eager):      # sizes the workspaces outside the capture
        rdk.rdk_verify_multi(p_static, q_static, C, 5, 0, cand_ids=cand_d, outputs=o)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(captured, n_cap, t_cap)
    rng = np.random.default_rng(6)
    for rep in range(3):
        perm = rng.permutation(B)
        p_static.copy_(dev(ragged["p"][:B][perm]))
        captured.token.fill_(-9)
        t_cap.fill_(-9)
        graph.replay()
        torch.cuda.synchronize()
        call(eager)
        n_e, t_e = rdk.rdk_tree_walk(child_d, eager.accepted, eager.token)
        torch.cuda.synchronize()
        for name in ("accepted", "token", "resid_mass"):
            assert torch.equal(getattr(captured, name), getattr(eager, name)), "replay %d: %s" % (rep, name)
        assert torch.equal(n_cap, n_e) and torch.equal(t_cap, t_e)
