"""ctypes front end of the fp64 CPU oracle (``rdk_oracle.c``).

TEST INFRASTRUCTURE ONLY.  The oracle is the slow, sequential, fp64 statement of
what Redistributing Drafter Kernels and the verification step of speculative
decoding compute (Alg. 1, Alg. 4, Eq. 1-3, Def. 2.1 of the paper).  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the GPU library never does, and this package never imports the GPU
library.  Every array that comes in is widened to fp64 first, so fp32 / bf16
inputs are taken at their exact values.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rdk_oracle.c")
_LIB = os.path.join(_HERE, "librdk_oracle.so")


def build(force=False):
    """Compile the oracle with gcc (plain C11, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", "-shared", "-fPIC",
             _SRC, "-o", _LIB, "-lm"])
        # the driver of the sanitizer test (tests/test_oracle_sanitizers.py builds it again with the sanitizers on)
        subprocess.check_call(
            ["gcc", "-O1", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", _SRC, os.path.join(_HERE, "sanitize_driver.c"),
             "-o", os.path.join(_HERE, "sanitize_driver.bin"), "-lm"])
    return _LIB


_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_I32 = ctypes.POINTER(ctypes.c_int32)
_U8 = ctypes.POINTER(ctypes.c_uint8)
_U32 = ctypes.POINTER(ctypes.c_uint32)
_i64 = ctypes.c_int64
_u64 = ctypes.c_uint64
_dbl = ctypes.c_double


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.orc_softmax.argtypes = [_D, _i64, _D]
        L.orc_softmax.restype = ctypes.c_int
        L.orc_tli.argtypes = [_D, _i64, _D]
        L.orc_tli.restype = ctypes.c_int
        L.orc_redistribute_dense.argtypes = [_D, _D, _i64, _i64, _D]
        L.orc_redistribute_dense.restype = None
        L.orc_redistribute_sparse.argtypes = [_D, _i64, _i64, _i64, _I32, _I32, _D, _D, _D]
        L.orc_redistribute_sparse.restype = None
        L.orc_taylor.argtypes = [_D, _D, _I32, _i64, _i64, _D, _D, _D]
        L.orc_taylor.restype = ctypes.c_int
        L.orc_features_from_scores.argtypes = [_D, _i64, _i64, _D]
        L.orc_features_from_scores.restype = None
        L.orc_overlap.argtypes = [_D, _D, _i64, _D, _D]
        L.orc_overlap.restype = None
        L.orc_kernel_l1.argtypes = [_D, _D, _i64]
        L.orc_kernel_l1.restype = _dbl
        L.orc_philox4x32_10.argtypes = [_U32, _U32, _U32]
        L.orc_philox4x32_10.restype = None
        L.orc_uniforms.argtypes = [_u64, _u64, _D]
        L.orc_uniforms.restype = None
        L.orc_sample_cdf.argtypes = [_D, _i64, _dbl]
        L.orc_sample_cdf.restype = _i64
        L.orc_accept.argtypes = [_dbl, _dbl, _dbl]
        L.orc_accept.restype = ctypes.c_int
        L.orc_sample_residual.argtypes = [_D, _D, _i64, _dbl]
        L.orc_sample_residual.restype = _i64
        L.orc_sequence_scan.argtypes = [_U8, _I32, _I32, _i64, _i64, _I32, _I32]
        L.orc_sequence_scan.restype = None
        L.orc_build_dense.argtypes = [_D, _i64, _i64, _I32, _i64, _dbl, _D]
        L.orc_build_dense.restype = ctypes.c_int
        L.orc_build_sparse.argtypes = [_D, _i64, _i64, _I32, _i64, _dbl, _i64, _I32, _D, _D, _D]
        L.orc_build_sparse.restype = ctypes.c_int
        L.orc_densify_sparse.argtypes = [_i64, _i64, _i64, _I32, _I32, _D, _D, _D]
        L.orc_densify_sparse.restype = None
        L.orc_verify_position.argtypes = [_D, _D, _i64, _u64, _u64, ctypes.c_int, _I32, _U8, _D, _D, _I32]
        L.orc_verify_position.restype = None
        L.orc_verify_multi.argtypes = [_D, _D, _i64, _i64, _u64, _u64, ctypes.c_int, _I32, _I32, _I32, _D]
        L.orc_verify_multi.restype = ctypes.c_int
        L.orc_tree_walk.argtypes = [_I32, _I32, _I32, _i64, _i64, _i64, _I32, _I32]
        L.orc_tree_walk.restype = None
        _lib = L
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _p(a, t):
    return a.ctypes.data_as(t)


# ----------------------------------------------------------------------------- per-vector steps
def softmax(z):
    z = _f64(z)
    out = np.empty_like(z)
    if lib().orc_softmax(_p(z, _D), z.size, _p(out, _D)) != 0:
        raise ValueError("softmax of an empty vector")
    return out


def tli(q_hat):
    """Eq. 1 on the kept slots: q_hat / sum(q_hat)."""
    q_hat = _f64(q_hat)
    out = np.empty_like(q_hat)
    if lib().orc_tli(_p(q_hat, _D), q_hat.size, _p(out, _D)) != 0:
        raise ValueError("TLI undefined: drafter mass on the kept ids is not positive")
    return out


def redistribute_dense(q_tli, M):
    """Alg. 1 step 2: p' = M^T q' with M of shape [n, N]."""
    q_tli, M = _f64(q_tli), _f64(M)
    n, N = M.shape
    assert q_tli.shape == (n,)
    out = np.empty(N)
    lib().orc_redistribute_dense(_p(q_tli, _D), _p(M, _D), n, N, _p(out, _D))
    return out


def redistribute_sparse(q_tli, N, kept_ids, nbr_idx, nbr_w, self_w):
    q_tli, kept_ids, nbr_idx = _f64(q_tli), _i32(kept_ids), _i32(nbr_idx)
    nbr_w, self_w = _f64(nbr_w), _f64(self_w)
    n = q_tli.size
    k = nbr_idx.shape[1] if nbr_idx.ndim == 2 else 0
    assert nbr_idx.shape == (N - n, k) and nbr_w.shape == (N - n, k) and self_w.shape == (n,)
    out = np.empty(N)
    lib().orc_redistribute_sparse(_p(q_tli, _D), n, N, k, _p(kept_ids, _I32), _p(nbr_idx, _I32),
                                  _p(nbr_w, _D), _p(self_w, _D), _p(out, _D))
    return out


def taylor(p, q_tli, kept_ids, return_scalars=False):
    """Eq. 3.  Returns p_Taylor (and theta, S = sum of the unnormalised vector)."""
    p, q_tli, kept_ids = _f64(p), _f64(q_tli), _i32(kept_ids)
    N, n = p.size, q_tli.size
    out = np.empty(N)
    th, S = _dbl(), _dbl()
    rc = lib().orc_taylor(_p(p, _D), _p(q_tli, _D), _p(kept_ids, _I32), n, N, _p(out, _D),
                          ctypes.byref(th), ctypes.byref(S))
    if rc != 0:
        raise ValueError("Eq. 3 undefined (rc=%d)" % rc)
    return (out, th.value, S.value) if return_scalars else out


def overlap(p, q):
    """(alpha, residual mass) = (sum min(p,q), sum (p - min(p,q)))  -- Def. 2.1, Alg. 4 step 8."""
    p, q = _f64(p), _f64(q)
    a, r = _dbl(), _dbl()
    lib().orc_overlap(_p(p, _D), _p(q, _D), p.size, ctypes.byref(a), ctypes.byref(r))
    return a.value, r.value


def kernel_l1(p, q):
    """||k||_1 for the drafter kernel of Def. 2.2."""
    p, q = _f64(p), _f64(q)
    return lib().orc_kernel_l1(_p(p, _D), _p(q, _D), p.size)


def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, _U32), _p(k, _U32), _p(out, _U32))
    return out


def uniforms(seed, index):
    u = np.empty(4)
    lib().orc_uniforms(int(seed), int(index), _p(u, _D))
    return u


def sample_cdf(w, u):
    w = _f64(w)
    return int(lib().orc_sample_cdf(_p(w, _D), w.size, float(u)))


def accept(u1, q_d, p_d):
    return bool(lib().orc_accept(float(u1), float(q_d), float(p_d)))


def sample_residual(p, q, u):
    p = _f64(p)
    qp = None
    if q is not None:
        q = _f64(q)
        qp = _p(q, _D)
    return int(lib().orc_sample_residual(_p(p, _D), qp, p.size, float(u)))


def sequence_scan(accept_flags, draft_ids, resid_ids, gamma):
    a = np.ascontiguousarray(accept_flags, dtype=np.uint8)
    d, r = _i32(draft_ids), _i32(resid_ids)
    S = a.size // gamma
    n_acc = np.empty(S, dtype=np.int32)
    out = np.empty((S, gamma + 1), dtype=np.int32)
    lib().orc_sequence_scan(_p(a, _U8), _p(d, _I32), _p(r, _I32), S, gamma, _p(n_acc, _I32), _p(out, _I32))
    return n_acc, out


# ----------------------------------------------------------------------------- kernel construction
def features_from_scores(z):
    """Sec. 3 (Omega estimated from data): z [T,N] sampled score rows -> centred token features F [N,T]; the cosine
    of two rows of F is the correlation of the two tokens' scores over the sample."""
    z = _f64(z)
    T, N = z.shape
    F = np.empty((N, T))
    lib().orc_features_from_scores(_p(z, _D), T, N, _p(F, _D))
    return F


def build_dense(E, kept_ids, tau):
    """Eq. 2 with Omega = cosine similarity of the rows of E.  Returns M [n, N] fp64."""
    E, kept_ids = _f64(E), _i32(kept_ids)
    N, d = E.shape
    n = kept_ids.size
    M = np.empty((n, N))
    if lib().orc_build_dense(_p(E, _D), N, d, _p(kept_ids, _I32), n, float(tau), _p(M, _D)) != 0:
        raise MemoryError
    return M


def build_sparse(E, kept_ids, tau, k, return_affinities=False):
    """Top-k sparse Eq. 2.  Returns (nbr_idx [N-n,k] int32, nbr_w [N-n,k], self_w [n])."""
    E, kept_ids = _f64(E), _i32(kept_ids)
    N, d = E.shape
    n = kept_ids.size
    nbr_idx = np.empty((N - n, k), dtype=np.int32)
    nbr_w = np.empty((N - n, k))
    self_w = np.empty(n)
    om = np.empty((N - n, k + 1))
    rc = lib().orc_build_sparse(_p(E, _D), N, d, _p(kept_ids, _I32), n, float(tau), k, _p(nbr_idx, _I32),
                                _p(nbr_w, _D), _p(self_w, _D), _p(om, _D))
    if rc != 0:
        raise ValueError("sparse build failed (rc=%d)" % rc)
    return (nbr_idx, nbr_w, self_w, om) if return_affinities else (nbr_idx, nbr_w, self_w)


def densify_sparse(N, kept_ids, nbr_idx, nbr_w, self_w):
    kept_ids, nbr_idx, nbr_w, self_w = _i32(kept_ids), _i32(nbr_idx), _f64(nbr_w), _f64(self_w)
    n = kept_ids.size
    k = nbr_idx.shape[1]
    M = np.empty((n, N))
    lib().orc_densify_sparse(n, N, k, _p(kept_ids, _I32), _p(nbr_idx, _I32), _p(nbr_w, _D), _p(self_w, _D),
                             _p(M, _D))
    return M


# ----------------------------------------------------------------------------- batched wrappers
def verify_batch(p, q_prime, seed, offset, sample_draft=True, draft_ids=None, gamma=0):
    """Alg. 4 steps 2, 4-8 for each row, then the per-sequence scan (steps 4-10) when gamma > 0.

    p [B,N]; q_prime [B,N] or None (bonus draw t ~ p only).  Position b uses Philox counter offset+b.
    """
    p = _f64(p)
    B, N = p.shape
    qp = None if q_prime is None else _f64(q_prime)
    d = np.full(B, -1, dtype=np.int32) if draft_ids is None else _i32(draft_ids).copy()
    acc = np.zeros(B, dtype=np.uint8)
    alpha, rmass = np.zeros(B), np.zeros(B)
    rid = np.full(B, -1, dtype=np.int32)
    L = lib()
    for b in range(B):
        a_, r_ = _dbl(), _dbl()
        L.orc_verify_position(_p(p[b], _D), None if qp is None else _p(qp[b], _D), N, int(seed), int(offset) + b,
                              1 if sample_draft else 0,
                              ctypes.cast(d.ctypes.data + 4 * b, _I32), ctypes.cast(acc.ctypes.data + b, _U8),
                              ctypes.byref(a_), ctypes.byref(r_), ctypes.cast(rid.ctypes.data + 4 * b, _I32))
        alpha[b], rmass[b] = a_.value, r_.value
    out = dict(draft_ids=d, accept=acc, alpha=alpha, resid_mass=rmass, resid_ids=rid)
    if gamma:
        out["n_accepted"], out["out_tokens"] = sequence_scan(acc, d, rid, gamma)
    return out


def verify_multi_batch(p, q_prime, C, seed, offset, cand_ids=None):
    """Several candidates per position (multi-step speculative sampling with q' as the drafter) for each row.

    cand_ids [B,C] given -> they are verified instead of drawn.  Returns a dict of cand_ids [B,C], accepted [B]
    (index of the accepted candidate, C if none), token [B], resid_mass [B,C]."""
    p, qp = _f64(p), _f64(q_prime)
    B, N = p.shape
    cand = np.full((B, C), -1, np.int32) if cand_ids is None else _i32(cand_ids).copy().reshape(B, C)
    acc, tok, rm = np.zeros(B, np.int32), np.zeros(B, np.int32), np.zeros((B, C))
    L = lib()
    for b in range(B):
        rc = L.orc_verify_multi(_p(p[b], _D), _p(qp[b], _D), N, C, int(seed), int(offset) + b, 1 if cand_ids is None else 0,
                                ctypes.cast(cand.ctypes.data + 4 * C * b, _I32), ctypes.cast(acc.ctypes.data + 4 * b, _I32),
                                ctypes.cast(tok.ctypes.data + 4 * b, _I32), ctypes.cast(rm.ctypes.data + 8 * C * b, _D))
        if rc != 0:
            raise MemoryError("orc_verify_multi")
    return dict(cand_ids=cand, accepted=acc, token=tok, resid_mass=rm)


def tree_walk(child_node, accepted, token, S, nodes, C):
    """Walk through S verified token trees of `nodes` nodes each; returns (n_accepted [S], out_tokens [S, nodes])."""
    cn, acc, tok = _i32(child_node).reshape(S * nodes * C), _i32(accepted), _i32(token)
    n_acc, out = np.zeros(S, np.int32), np.zeros((S, nodes), np.int32)
    lib().orc_tree_walk(_p(cn, _I32), _p(acc, _I32), _p(tok, _I32), S, nodes, C, _p(n_acc, _I32), _p(out, _I32))
    return n_acc, out


def multi_uniform(seed, index, m):
    """The m-th uniform of a position in the multi-candidate stream: word m % 4 of Philox(counter=(index, m // 4, 0))."""
    w = philox4x32_10([index & 0xFFFFFFFF, (index >> 32) & 0xFFFFFFFF, m // 4, 0], [seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF])
    return float(int(w[m % 4]) >> 8) / 16777216.0


def probs_from(x, kind):
    """Rows of x as probabilities: kind 'prob' passes through, 'logit' applies the softmax."""
    x = _f64(x)
    if kind == "prob":
        return x
    return np.stack([softmax(r) for r in x])


def redistribute_batch(mode, q, kept_ids, N, p=None, M=None, sparse=None):
    """Alg. 1 steps 1-2 for each row of q [B,n] (non-negative, not necessarily normalised).

    mode: 'exact' (needs M [n,N]), 'sparse' (needs sparse=(nbr_idx, nbr_w, self_w)),
    'taylor' (needs p [B,N]), 'tli' (identity kernel: scatter of q').
    """
    q = _f64(q)
    out = np.empty((q.shape[0], N))
    for b in range(q.shape[0]):
        qt = tli(q[b])
        if mode == "exact":
            out[b] = redistribute_dense(qt, M)
        elif mode == "sparse":
            out[b] = redistribute_sparse(qt, N, kept_ids, *sparse)
        elif mode == "taylor":
            out[b] = taylor(p[b], qt, kept_ids)
        elif mode == "tli":
            out[b] = 0.0
            out[b, np.asarray(kept_ids)] = qt
        else:
            raise ValueError(mode)
    return out
