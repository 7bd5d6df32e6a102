"""ctypes binding of the RDK HIP library (``librdk_hip.so``): argument marshalling only.

Function names and arguments mirror ``include/rdk.h``.  Tensors are torch CUDA (ROCm) tensors; torch is
used for device memory and streams, nothing else: every step of the path runs in the library's kernels.
Loading fails loudly if the library has not been built (``python -m paper_2506_03206_amd.build``);
there is no fallback path.
"""
import ctypes
import os

import torch  # noqa: F401  (imported first so that the HIP runtime already in the process is shared)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librdk_hip.so")

OK = 0
DENSE_F32, DENSE_BF16, SPARSE_TOPK, IDENTITY = 0, 1, 2, 3
PROB_F32, LOGIT_F32, LOGIT_BF16 = 0, 1, 2
LINEAR_TAYLOR, LINEAR_SPARSE = 0, 1

EXPORTS = [
    "rdk_status_string", "rdk_last_hip_error", "rdk_kernel_storage_bytes", "rdk_build_kernel", "rdk_destroy_kernel",
    "rdk_kernel_get_sparse", "rdk_kernel_get_dense", "rdk_workspace_bytes", "rdk_redistribute_exact",
    "rdk_redistribute_linear", "rdk_verify_workspace_bytes", "rdk_verify_sample", "rdk_philox_words",
    "rdk_timing_select", "rdk_timing_read", "rdk_redistribute_verify_workspace_bytes", "rdk_redistribute_verify",
    "rdk_sample_draft_workspace_bytes", "rdk_sample_draft", "rdk_features_from_scores",
    "rdk_verify_multi_workspace_bytes", "rdk_verify_multi", "rdk_tree_walk", "rdk_verify_sample_static",
]


class KernelDesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("n", ctypes.c_int32), ("d", ctypes.c_int32), ("k", ctypes.c_int32),
                ("kept_ids", ctypes.c_void_p), ("embeddings", ctypes.c_void_p), ("dense_M", ctypes.c_void_p),
                ("sparse_idx", ctypes.c_void_p), ("sparse_w", ctypes.c_void_p), ("self_w", ctypes.c_void_p),
                ("tau", ctypes.c_float), ("format", ctypes.c_int), ("validate", ctypes.c_int32)]


class VerifyDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("N", ctypes.c_int32), ("gamma", ctypes.c_int32),
                ("sample_draft", ctypes.c_int32), ("seed", ctypes.c_uint64), ("offset", ctypes.c_uint64)]


class MultiDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("N", ctypes.c_int32), ("C", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("offset", ctypes.c_uint64), ("sample_candidates", ctypes.c_int)]


class RdkError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().rdk_status_string(status).decode()
        if status == 8:
            msg += " (" + lib().rdk_last_hip_error().decode() + ")"
        super().__init__("%s: %s [status %d]" % (where, msg, status))


_lib = None


def lib():
    """The loaded C library (raises if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: build it with `python -m paper_2506_03206_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        psz = ctypes.POINTER(ctypes.c_size_t)
        L.rdk_status_string.restype = ctypes.c_char_p
        L.rdk_status_string.argtypes = [ctypes.c_int]
        L.rdk_last_hip_error.restype = ctypes.c_char_p
        L.rdk_last_hip_error.argtypes = []
        L.rdk_kernel_storage_bytes.argtypes = [ctypes.POINTER(KernelDesc), psz, psz]
        L.rdk_build_kernel.argtypes = [ctypes.POINTER(KernelDesc), vp, sz, vp, sz, vp, ctypes.POINTER(vp)]
        L.rdk_destroy_kernel.argtypes = [vp]
        L.rdk_kernel_get_sparse.argtypes = [vp, vp, vp, vp, vp]
        L.rdk_kernel_get_dense.argtypes = [vp, vp, i64, vp]
        L.rdk_workspace_bytes.argtypes = [vp, i32, psz]
        L.rdk_redistribute_exact.argtypes = [vp, vp, ctypes.c_int, i64, i32, vp, i64, vp, sz, vp]
        L.rdk_redistribute_linear.argtypes = [vp, ctypes.c_int, vp, ctypes.c_int, i64, vp, ctypes.c_int, i64, i32, vp, i64,
                                              vp, sz, vp]
        L.rdk_verify_workspace_bytes.argtypes = [ctypes.POINTER(VerifyDesc), psz]
        L.rdk_verify_sample.argtypes = [ctypes.POINTER(VerifyDesc), vp, ctypes.c_int, i64, vp, i64, vp, vp, vp, vp, vp, vp,
                                        vp, vp, sz, vp]
        L.rdk_verify_sample_static.argtypes = [ctypes.POINTER(VerifyDesc), vp, ctypes.c_int, i64, vp, i64, vp, vp, vp, vp, vp,
                                               vp, vp, vp]
        L.rdk_philox_words.argtypes = [ctypes.c_uint64, ctypes.c_uint64, i32, vp, vp]
        L.rdk_redistribute_verify_workspace_bytes.argtypes = [vp, ctypes.c_int, ctypes.POINTER(VerifyDesc), psz]
        L.rdk_redistribute_verify.argtypes = [vp, ctypes.c_int, ctypes.POINTER(VerifyDesc), vp, ctypes.c_int, i64, vp,
                                              ctypes.c_int, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.rdk_sample_draft_workspace_bytes.argtypes = [vp, i32, psz]
        L.rdk_sample_draft.argtypes = [vp, vp, ctypes.c_int, i64, i32, ctypes.c_uint64, ctypes.c_uint64, vp, vp, vp, i64, vp, sz, vp]
        L.rdk_features_from_scores.argtypes = [vp, ctypes.c_int, i64, i32, i32, vp, i64, vp]
        L.rdk_verify_multi_workspace_bytes.argtypes = [ctypes.POINTER(MultiDesc), ctypes.c_int, psz]
        L.rdk_verify_multi.argtypes = [ctypes.POINTER(MultiDesc), vp, ctypes.c_int, i64, vp, i64, vp, vp, vp, vp, vp, sz, vp]
        L.rdk_tree_walk.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.rdk_timing_select.argtypes = [ctypes.c_char_p]
        L.rdk_timing_read.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)]
        for name in EXPORTS:
            # without declared argument types ctypes pushes 4-byte ints for 64-bit stack parameters
            assert getattr(L, name).argtypes is not None, "argtypes missing for " + name
            if name not in ("rdk_status_string", "rdk_last_hip_error"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status, where):
    if status != OK:
        raise RdkError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _kind_of(t, kind):
    """Input kind of a tensor: 'prob' | 'logit' decided by the caller, bf16 by dtype."""
    if kind == "prob":
        assert t.dtype == torch.float32
        return PROB_F32
    if t.dtype == torch.bfloat16:
        return LOGIT_BF16
    assert t.dtype == torch.float32
    return LOGIT_F32


def _rows(t):
    assert t.dim() == 2 and t.stride(1) == 1 and t.is_cuda
    return t.stride(0)


class Kernel:
    """A built token-affinity kernel M (owns its device storage; see rdk_build_kernel)."""

    def __init__(self, handle, storage, N, n, k, fmt):
        self.handle, self.storage, self.N, self.n, self.k, self.format = handle, storage, N, n, k, fmt
        self._ws = None

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.rdk_destroy_kernel(self.handle)
            self.handle = None

    def workspace(self, B):
        need = ctypes.c_size_t()
        _check(lib().rdk_workspace_bytes(self.handle, B, ctypes.byref(need)), "rdk_workspace_bytes")
        if self._ws is None or self._ws.numel() < need.value:
            self._ws = torch.empty(need.value, dtype=torch.uint8, device=self.storage.device)
        return self._ws


def rdk_features_from_scores(z, kind="logit"):
    """Centred token features [N, T] from T sampled score rows z [T, N] (fp32, or bf16 logits): embeddings whose
    cosine is the correlation of the tokens' scores over the sample."""
    T, N = z.shape
    F = torch.empty((N, T), dtype=torch.float32, device=z.device)
    _check(lib().rdk_features_from_scores(_ptr(z), _kind_of(z, kind), _rows(z), T, N, _ptr(F), T, _stream()),
           "rdk_features_from_scores")
    return F


def rdk_build_kernel(N, kept_ids, fmt, embeddings=None, tau=0.1, k=0, dense_M=None, sparse=None, validate=True):
    """Eq. 2 of the paper on the device.  kept_ids int32 [n]; embeddings fp32 [N,d] or a finished kernel."""
    dev = kept_ids.device
    assert kept_ids.dtype == torch.int32 and kept_ids.is_contiguous()
    d = KernelDesc()
    d.N, d.n, d.k, d.format, d.tau, d.validate = N, kept_ids.numel(), k, fmt, tau, 1 if validate else 0
    d.kept_ids = kept_ids.data_ptr()
    keep = [kept_ids]
    if embeddings is not None:
        assert embeddings.dtype == torch.float32 and embeddings.is_contiguous() and embeddings.shape[0] == N
        d.embeddings, d.d = embeddings.data_ptr(), embeddings.shape[1]
        keep.append(embeddings)
    if dense_M is not None:
        assert dense_M.dtype == torch.float32 and dense_M.is_contiguous() and dense_M.shape == (d.n, N)
        d.dense_M = dense_M.data_ptr()
        keep.append(dense_M)
    if sparse is not None:
        idx, w, self_w = sparse
        assert idx.dtype == torch.int32 and w.dtype == torch.float32 and self_w.dtype == torch.float32
        assert idx.is_contiguous() and w.is_contiguous() and self_w.is_contiguous()
        assert idx.shape == (N - d.n, k) and w.shape == idx.shape and self_w.shape == (d.n,)
        d.sparse_idx, d.sparse_w, d.self_w = idx.data_ptr(), w.data_ptr(), self_w.data_ptr()
        keep += [idx, w, self_w]
    sb, wb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().rdk_kernel_storage_bytes(ctypes.byref(d), ctypes.byref(sb), ctypes.byref(wb)), "rdk_kernel_storage_bytes")
    storage = torch.empty(sb.value, dtype=torch.uint8, device=dev)
    ws = torch.empty(wb.value, dtype=torch.uint8, device=dev)
    h = ctypes.c_void_p()
    _check(lib().rdk_build_kernel(ctypes.byref(d), _ptr(storage), sb.value, _ptr(ws), wb.value, _stream(), ctypes.byref(h)),
           "rdk_build_kernel")
    torch.cuda.current_stream().synchronize()   # the build scratch and the inputs may be released after this
    return Kernel(h, storage, N, d.n, k, fmt)


def rdk_kernel_get_sparse(kernel):
    dev = kernel.storage.device
    idx = torch.empty((kernel.N - kernel.n, kernel.k), dtype=torch.int32, device=dev)
    w = torch.empty((kernel.N - kernel.n, kernel.k), dtype=torch.float32, device=dev)
    self_w = torch.empty(kernel.n, dtype=torch.float32, device=dev)
    _check(lib().rdk_kernel_get_sparse(kernel.handle, _ptr(idx), _ptr(w), _ptr(self_w), _stream()), "rdk_kernel_get_sparse")
    return idx, w, self_w


def rdk_kernel_get_dense(kernel):
    M = torch.empty((kernel.n, kernel.N), dtype=torch.float32, device=kernel.storage.device)
    _check(lib().rdk_kernel_get_dense(kernel.handle, _ptr(M), kernel.N, _stream()), "rdk_kernel_get_dense")
    return M


def rdk_redistribute_exact(kernel, q, q_kind="prob", out=None):
    B = q.shape[0]
    out = torch.empty((B, kernel.N), dtype=torch.float32, device=q.device) if out is None else out
    ws = kernel.workspace(B)
    _check(lib().rdk_redistribute_exact(kernel.handle, _ptr(q), _kind_of(q, q_kind), _rows(q), B, _ptr(out), _rows(out),
                                        _ptr(ws), ws.numel(), _stream()), "rdk_redistribute_exact")
    return out


def rdk_redistribute_linear(kernel, mode, q, q_kind="prob", p=None, p_kind="prob", out=None):
    B = q.shape[0]
    out = torch.empty((B, kernel.N), dtype=torch.float32, device=q.device) if out is None else out
    ws = kernel.workspace(B)
    pk, ldp = (PROB_F32, 0) if p is None else (_kind_of(p, p_kind), _rows(p))
    _check(lib().rdk_redistribute_linear(kernel.handle, mode, _ptr(p), pk, ldp, _ptr(q), _kind_of(q, q_kind), _rows(q), B,
                                         _ptr(out), _rows(out), _ptr(ws), ws.numel(), _stream()),
           "rdk_redistribute_linear")
    return out


class VerifyOutputs:
    """Output buffers (and scratch) of rdk_verify_sample for a fixed batch shape; reusable across calls."""

    def __init__(self, B, N, gamma, device):
        self.B, self.N, self.gamma = B, N, gamma
        self.draft_ids = torch.full((B,), -1, dtype=torch.int32, device=device)
        self.accept = torch.zeros(B, dtype=torch.uint8, device=device)
        self.alpha = torch.zeros(B, dtype=torch.float32, device=device)
        self.resid_mass = torch.zeros(B, dtype=torch.float32, device=device)
        self.resid_ids = torch.full((B,), -1, dtype=torch.int32, device=device)
        S = B // gamma if gamma else 0
        self.n_accepted = torch.zeros(S, dtype=torch.int32, device=device) if gamma else None
        self.out_tokens = torch.zeros((S, gamma + 1), dtype=torch.int32, device=device) if gamma else None
        d = VerifyDesc(B=B, N=N, gamma=gamma, sample_draft=1, seed=0, offset=0)
        need = ctypes.c_size_t()
        _check(lib().rdk_verify_workspace_bytes(ctypes.byref(d), ctypes.byref(need)), "rdk_verify_workspace_bytes")
        self.ws = torch.empty(need.value, dtype=torch.uint8, device=device)


def rdk_verify_sample(p, q_prime, seed, offset=0, gamma=0, p_kind="prob", draft_ids=None, outputs=None):
    """Alg. 4 steps 2, 4-10 for every row.  draft_ids given -> they are verified instead of sampled."""
    B, N = p.shape
    o = outputs or VerifyOutputs(B, N, gamma, p.device)
    assert (o.B, o.N, o.gamma) == (B, N, gamma)
    if draft_ids is not None:
        o.draft_ids.copy_(draft_ids)
    d = VerifyDesc(B=B, N=N, gamma=gamma, sample_draft=0 if draft_ids is not None else 1, seed=seed, offset=offset)
    ldq = 0 if q_prime is None else _rows(q_prime)
    _check(lib().rdk_verify_sample(ctypes.byref(d), _ptr(p), _kind_of(p, p_kind), _rows(p), _ptr(q_prime), ldq,
                                   _ptr(o.draft_ids), _ptr(o.accept), _ptr(o.alpha), _ptr(o.resid_mass), _ptr(o.resid_ids),
                                   _ptr(o.n_accepted), _ptr(o.out_tokens), _ptr(o.ws), o.ws.numel(), _stream()),
           "rdk_verify_sample")
    return o


def rdk_verify_sample_static(p, q_prime, seed, offset=0, gamma=0, p_kind="prob", draft_ids=None, outputs=None):
    """rdk_verify_sample without a workspace: the scratch is a fixed device array inside the library.  `outputs` must
    be given (the call itself allocates nothing); its own workspace tensor is not used."""
    B, N = p.shape
    o = outputs
    assert o is not None and (o.B, o.N, o.gamma) == (B, N, gamma)
    if draft_ids is not None:
        o.draft_ids.copy_(draft_ids)
    d = VerifyDesc(B=B, N=N, gamma=gamma, sample_draft=0 if draft_ids is not None else 1, seed=seed, offset=offset)
    ldq = 0 if q_prime is None else _rows(q_prime)
    _check(lib().rdk_verify_sample_static(ctypes.byref(d), _ptr(p), _kind_of(p, p_kind), _rows(p), _ptr(q_prime), ldq,
                                          _ptr(o.draft_ids), _ptr(o.accept), _ptr(o.alpha), _ptr(o.resid_mass),
                                          _ptr(o.resid_ids), _ptr(o.n_accepted), _ptr(o.out_tokens), _stream()),
           "rdk_verify_sample_static")
    return o


def rdk_redistribute_verify(kernel, mode, p, q, seed, offset=0, gamma=0, p_kind="prob", q_kind="prob", draft_ids=None,
                            outputs=None, q_prime=None):
    """Fused rdk_redistribute_linear + rdk_verify_sample.  q_prime: optional [B,N] tensor that receives q'."""
    B, N = p.shape
    o = outputs or VerifyOutputs(B, N, gamma, p.device)
    assert (o.B, o.N, o.gamma) == (B, N, gamma)
    if draft_ids is not None:
        o.draft_ids.copy_(draft_ids)
    d = VerifyDesc(B=B, N=N, gamma=gamma, sample_draft=0 if draft_ids is not None else 1, seed=seed, offset=offset)
    need = ctypes.c_size_t()
    _check(lib().rdk_redistribute_verify_workspace_bytes(kernel.handle, mode, ctypes.byref(d), ctypes.byref(need)),
           "rdk_redistribute_verify_workspace_bytes")
    if getattr(o, "fused_ws", None) is None or o.fused_ws.numel() < need.value:
        o.fused_ws = torch.empty(need.value, dtype=torch.uint8, device=p.device)
    ldo = 0 if q_prime is None else _rows(q_prime)
    _check(lib().rdk_redistribute_verify(kernel.handle, mode, ctypes.byref(d), _ptr(p), _kind_of(p, p_kind), _rows(p),
                                         _ptr(q), _kind_of(q, q_kind), _rows(q), _ptr(q_prime), ldo, _ptr(o.draft_ids),
                                         _ptr(o.accept), _ptr(o.alpha), _ptr(o.resid_mass), _ptr(o.resid_ids),
                                         _ptr(o.n_accepted), _ptr(o.out_tokens), _ptr(o.fused_ws), o.fused_ws.numel(),
                                         _stream()), "rdk_redistribute_verify")
    return o


def rdk_sample_draft(kernel, q, seed, offset=0, q_kind="prob", q_prime=None, draft_ids=None, q_draft=None):
    """Draft tokens drawn from q' = M^T TLI(q) before any target row exists.  Returns (draft_ids [B] int32,
    q_draft [B] fp32 = q' at the drafted id).  q_prime: [B,N] tensor that receives the rows (required unless the
    kernel is a top-k sparse one)."""
    B = q.shape[0]
    if draft_ids is None:
        draft_ids = torch.empty(B, dtype=torch.int32, device=q.device)
    if q_draft is None:
        q_draft = torch.empty(B, dtype=torch.float32, device=q.device)
    need = ctypes.c_size_t()
    _check(lib().rdk_sample_draft_workspace_bytes(kernel.handle, B, ctypes.byref(need)), "rdk_sample_draft_workspace_bytes")
    if getattr(kernel, "_draft_ws", None) is None or kernel._draft_ws.numel() < need.value:
        kernel._draft_ws = torch.empty(need.value, dtype=torch.uint8, device=q.device)
    ldo = 0 if q_prime is None else _rows(q_prime)
    _check(lib().rdk_sample_draft(kernel.handle, _ptr(q), _kind_of(q, q_kind), _rows(q), B, seed, offset, _ptr(draft_ids),
                                  _ptr(q_draft), _ptr(q_prime), ldo, _ptr(kernel._draft_ws), kernel._draft_ws.numel(),
                                  _stream()), "rdk_sample_draft")
    return draft_ids, q_draft


class MultiOutputs:
    """Outputs of rdk_verify_multi: cand_ids [B,C], accepted [B], token [B], resid_mass [B,C]."""

    def __init__(self, B, C, device):
        self.cand_ids = torch.full((B, C), -1, dtype=torch.int32, device=device)
        self.accepted = torch.zeros(B, dtype=torch.int32, device=device)
        self.token = torch.full((B,), -1, dtype=torch.int32, device=device)
        self.resid_mass = torch.zeros((B, C), dtype=torch.float32, device=device)
        self.ws = None


def rdk_verify_multi(p, q_prime, C, seed, offset=0, p_kind="prob", cand_ids=None, outputs=None):
    """Several candidates per position: kept candidate (or the residual draw) for every row.
    cand_ids [B,C] given -> they are verified instead of drawn from q_prime."""
    B, N = p.shape
    o = outputs or MultiOutputs(B, C, p.device)
    if cand_ids is not None:
        o.cand_ids.copy_(cand_ids.reshape(B, C))
    d = MultiDesc(B=B, N=N, C=C, seed=seed, offset=offset, sample_candidates=0 if cand_ids is not None else 1)
    kind = _kind_of(p, p_kind)
    need = ctypes.c_size_t()
    _check(lib().rdk_verify_multi_workspace_bytes(ctypes.byref(d), kind, ctypes.byref(need)), "rdk_verify_multi_workspace_bytes")
    if o.ws is None or o.ws.numel() < need.value:
        o.ws = torch.empty(need.value, dtype=torch.uint8, device=p.device)
    _check(lib().rdk_verify_multi(ctypes.byref(d), _ptr(p), kind, _rows(p), _ptr(q_prime), _rows(q_prime), _ptr(o.cand_ids),
                                  _ptr(o.accepted), _ptr(o.token), _ptr(o.resid_mass), _ptr(o.ws), o.ws.numel(), _stream()),
           "rdk_verify_multi")
    return o


def rdk_tree_walk(child_node, accepted, token):
    """Walk through verified token trees.  child_node [S, nodes, C] int32; accepted, token [S * nodes] from
    rdk_verify_multi on the nodes.  Returns (n_accepted [S], out_tokens [S, nodes])."""
    S, nodes, C = child_node.shape
    assert child_node.is_contiguous() and accepted.numel() == S * nodes and token.numel() == S * nodes
    n_acc = torch.zeros(S, dtype=torch.int32, device=child_node.device)
    out = torch.full((S, nodes), -1, dtype=torch.int32, device=child_node.device)
    _check(lib().rdk_tree_walk(S, nodes, C, _ptr(child_node), _ptr(accepted), _ptr(token), _ptr(n_acc), _ptr(out), _stream()),
           "rdk_tree_walk")
    return n_acc, out


def rdk_philox_words(seed, offset, count, device="cuda"):
    words = torch.empty((count, 4), dtype=torch.int32, device=device)
    _check(lib().rdk_philox_words(seed, offset, count, _ptr(words), _stream()), "rdk_philox_words")
    return words


def rdk_timing_select(kernel_name):
    """Bracket launches of one library kernel ('*' = all hot-path kernels, None = off) with HIP events."""
    _check(lib().rdk_timing_select(kernel_name.encode() if kernel_name else None), "rdk_timing_select")


def rdk_timing_read(kernel_name):
    """(launches, total milliseconds) recorded for a kernel since the last read."""
    n, ms = ctypes.c_int64(), ctypes.c_double()
    _check(lib().rdk_timing_read(kernel_name.encode(), ctypes.byref(n), ctypes.byref(ms)), "rdk_timing_read")
    return n.value, ms.value
