"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares, and its
argument validation and size queries behave (no kernel is launched, so no GPU is needed)."""
import ctypes
import os
import re

import pytest

from conftest import ROOT


@pytest.fixture(scope="module")
def rdk():
    from paper_2506_03206_amd import rdk as mod
    if not os.path.exists(mod.LIB_PATH):
        from paper_2506_03206_amd import build
        build.build()
    return mod


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rdk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rdk_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(rdk):
    names = declared_symbols()
    assert "rdk_build_kernel" in names and "rdk_redistribute_exact" in names
    assert "rdk_redistribute_linear" in names and "rdk_verify_sample" in names
    L = rdk.lib()
    for name in names:
        assert hasattr(L, name), name
    assert sorted(rdk.EXPORTS) == names


def test_status_strings(rdk):
    L = rdk.lib()
    seen = {L.rdk_status_string(i).decode() for i in range(10)}
    assert len(seen) == 10 and "ok" in seen
    assert L.rdk_status_string(99).decode() == "unknown status"
    assert L.rdk_last_hip_error().decode() == ""


def _desc(rdk, **kw):
    d = rdk.KernelDesc()
    d.N, d.n, d.d, d.k, d.tau, d.format, d.validate = 1024, 256, 64, 8, 0.1, rdk.SPARSE_TOPK, 0
    d.kept_ids, d.embeddings = 0x1000, 0x2000          # never dereferenced by the size query
    for key, val in kw.items():
        setattr(d, key, val)
    return d


def test_storage_query_and_validation(rdk):
    L = rdk.lib()
    sb, wb = ctypes.c_size_t(), ctypes.c_size_t()
    q = lambda d: L.rdk_kernel_storage_bytes(ctypes.byref(d), ctypes.byref(sb), ctypes.byref(wb))
    assert q(_desc(rdk)) == 0
    up = lambda x: (x + 255) // 256 * 256
    # kept ids, slot table, pruned ids, first slot per 1024-id chunk, lane map (64 records of 8 bytes per chunk), first
    # piece per chunk, the pieces of at most 64 kept slots (one per chunk and one per 64 slots at most, 8 bytes each)
    head = 1024 + 4096 + up(769 * 4) + up(2 * 4) + up(1 * 64 * 8) + up(2 * 4) + up((1 + 256 // 64 + 1) * 8)
    # [N-n, 16] (slot, weight) pairs (k = 8 padded to 16 entries) and the diagonal weights
    assert sb.value == head + up(768 * 16 * 8 + 512) + 1024
    assert q(_desc(rdk, format=rdk.DENSE_F32)) == 0 and sb.value == head + 256 * 1024 * 4
    assert q(_desc(rdk, format=rdk.DENSE_BF16)) == 0 and sb.value == head + 384 * 1024 * 2 + 1024
    assert wb.value > 256 * 1024 * 4                       # the fp32 matrix that gets packed
    assert q(_desc(rdk, format=rdk.IDENTITY, embeddings=None)) == 0 and sb.value == head
    assert q(_desc(rdk, n=0)) == 2 and q(_desc(rdk, n=2000)) == 2 and q(_desc(rdk, k=65)) == 2
    assert q(_desc(rdk, kept_ids=None)) == 1 and q(_desc(rdk, embeddings=None)) == 1
    assert q(_desc(rdk, tau=0.0)) == 2 and q(_desc(rdk, format=7)) == 3
    assert q(_desc(rdk, kept_ids=0x1004)) == 9
    assert L.rdk_kernel_storage_bytes(None, ctypes.byref(sb), ctypes.byref(wb)) == 1
    # a supplied sparse kernel needs all three tables
    assert q(_desc(rdk, embeddings=None, self_w=0x3000)) == 1
    assert q(_desc(rdk, embeddings=None, self_w=0x3000, sparse_idx=0x4000, sparse_w=0x5000)) == 0


def test_verify_argument_checks(rdk):
    L = rdk.lib()
    need = ctypes.c_size_t()
    d = rdk.VerifyDesc(B=256, N=128256, gamma=8, sample_draft=1, seed=1, offset=0)
    assert L.rdk_verify_workspace_bytes(ctypes.byref(d), ctypes.byref(need)) == 0
    nchunks = (128256 + 1023) // 1024
    assert need.value >= 3 * 256 * nchunks * 4
    bad = rdk.VerifyDesc(B=10, N=64, gamma=4, sample_draft=1, seed=1, offset=0)
    assert L.rdk_verify_workspace_bytes(ctypes.byref(bad), ctypes.byref(need)) == 2        # B % gamma != 0
    vp = ctypes.c_void_p
    args = lambda p=0x1000, q=0x2000, draft=0x3000, acc=0x4000, rid=0x5000, ws=0x6000, wsb=1 << 30, ldp=128256, kind=0: (
        ctypes.byref(d), vp(p), kind, ldp, vp(q), 128256, vp(draft), vp(acc), None, None, vp(rid), None, None, vp(ws), wsb, None)
    assert L.rdk_verify_sample(*args(p=None)) == 1
    assert L.rdk_verify_sample(*args(acc=None)) == 1
    assert L.rdk_verify_sample(*args(ldp=100)) == 2
    assert L.rdk_verify_sample(*args(kind=5)) == 3
    assert L.rdk_verify_sample(*args(p=0x1004)) == 9
    assert L.rdk_verify_sample(*args(wsb=16)) == 6
    assert L.rdk_verify_sample(*args(q=None)) == 7                                       # bonus draw cannot be scanned
    assert L.rdk_philox_words(1, 0, 0, vp(0x1000), None) == 2
    assert L.rdk_redistribute_exact(None, vp(0x1000), 0, 10, 1, vp(0x2000), 10, vp(0x3000), 10, None) == 1


def test_draft_and_feature_argument_checks(rdk):
    """The newer entry points validate on the host too (nothing is launched)."""
    L = rdk.lib()
    vp = ctypes.c_void_p
    need = ctypes.c_size_t()
    assert L.rdk_sample_draft_workspace_bytes(None, 8, ctypes.byref(need)) == 1
    assert L.rdk_sample_draft(None, vp(0x1000), 0, 16, 8, 1, 0, vp(0x2000), None, None, 0, vp(0x3000), 1 << 20, None) == 1
    feat = lambda z=0x1000, kind=1, ldz=100, T=8, N=100, F=0x2000, ldf=8: L.rdk_features_from_scores(
        vp(z) if z else None, kind, ldz, T, N, vp(F) if F else None, ldf, None)
    assert feat(z=None) == 1 and feat(F=None) == 1
    assert feat(kind=4) == 3
    assert feat(T=1) == 2 and feat(ldz=99) == 2 and feat(ldf=7) == 2 and feat(N=0) == 2
    assert feat(z=0x1008) == 9 and feat(F=0x2004) == 9


def test_multi_candidate_argument_checks(rdk):
    L = rdk.lib()
    vp = ctypes.c_void_p
    need = ctypes.c_size_t()
    d = rdk.MultiDesc(B=256, N=128256, C=4, seed=1, offset=0, sample_candidates=1)
    assert L.rdk_verify_multi_workspace_bytes(ctypes.byref(d), 0, ctypes.byref(need)) == 0 and need.value >= 256
    assert L.rdk_verify_multi_workspace_bytes(ctypes.byref(d), 2, ctypes.byref(need)) == 0 and need.value >= 256 * 8
    assert L.rdk_verify_multi_workspace_bytes(ctypes.byref(d), 7, ctypes.byref(need)) == 3
    assert L.rdk_verify_multi_workspace_bytes(None, 0, ctypes.byref(need)) == 1
    for field, value, status in (("C", 0, 2), ("C", 17, 7), ("B", 0, 2), ("N", 0, 2), ("N", (1 << 21) + 1, 7)):
        bad = rdk.MultiDesc(B=256, N=128256, C=4, seed=1, offset=0, sample_candidates=1)
        setattr(bad, field, value)
        assert L.rdk_verify_multi_workspace_bytes(ctypes.byref(bad), 0, ctypes.byref(need)) == status, field
    args = lambda p=0x1000, q=0x2000, cand=0x3000, acc=0x4000, tok=0x5000, ws=0x6000, wsb=1 << 20, ldp=128256, ldq=128256, kind=0: (
        ctypes.byref(d), vp(p) if p else None, kind, ldp, vp(q) if q else None, ldq, vp(cand) if cand else None,
        vp(acc) if acc else None, vp(tok) if tok else None, None, vp(ws) if ws else None, wsb, None)
    assert L.rdk_verify_multi(*args(p=None)) == 1 and L.rdk_verify_multi(*args(q=None)) == 1
    assert L.rdk_verify_multi(*args(cand=None)) == 1 and L.rdk_verify_multi(*args(tok=None)) == 1
    assert L.rdk_verify_multi(*args(ldp=100)) == 2 and L.rdk_verify_multi(*args(ldq=100)) == 2
    assert L.rdk_verify_multi(*args(kind=5)) == 3
    assert L.rdk_verify_multi(*args(p=0x1004)) == 9 and L.rdk_verify_multi(*args(q=0x2008)) == 9
    assert L.rdk_verify_multi(*args(wsb=16)) == 6
    walk = lambda S=4, nodes=5, C=2, child=0x1000, acc=0x2000, tok=0x3000, n=0x4000, out=0x5000: L.rdk_tree_walk(
        S, nodes, C, vp(child) if child else None, vp(acc) if acc else None, vp(tok) if tok else None, vp(n) if n else None,
        vp(out) if out else None, None)
    assert walk(S=0) == 2 and walk(nodes=0) == 2 and walk(C=0) == 2
    assert walk(child=None) == 1 and walk(acc=None) == 1 and walk(tok=None) == 1 and walk(n=None) == 1 and walk(out=None) == 1


def test_descriptor_layouts_match_the_header(rdk, tmp_path):
    """The ctypes mirrors of the descriptor structs against the C compiler's view of include/rdk.h."""
    import subprocess
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "rdk.h"\n'
                   '#define F(T, f) printf(#T "." #f " %zu\\n", offsetof(T, f));\n'
                   'int main(void) {\n'
                   '  printf("rdk_verify_desc_t %zu\\n", sizeof(rdk_verify_desc_t));\n'
                   '  F(rdk_verify_desc_t, B) F(rdk_verify_desc_t, N) F(rdk_verify_desc_t, gamma) F(rdk_verify_desc_t, sample_draft)\n'
                   '  F(rdk_verify_desc_t, seed) F(rdk_verify_desc_t, offset)\n'
                   '  printf("rdk_multi_desc_t %zu\\n", sizeof(rdk_multi_desc_t));\n'
                   '  F(rdk_multi_desc_t, B) F(rdk_multi_desc_t, N) F(rdk_multi_desc_t, C) F(rdk_multi_desc_t, seed)\n'
                   '  F(rdk_multi_desc_t, offset) F(rdk_multi_desc_t, sample_candidates)\n'
                   '  printf("rdk_kernel_desc_t %zu\\n", sizeof(rdk_kernel_desc_t));\n'
                   '  F(rdk_kernel_desc_t, kept_ids) F(rdk_kernel_desc_t, self_w) F(rdk_kernel_desc_t, tau) F(rdk_kernel_desc_t, format)\n'
                   '  F(rdk_kernel_desc_t, validate)\n  return 0;\n}\n')
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = dict(line.rsplit(" ", 1) for line in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.splitlines())
    mirrors = {"rdk_verify_desc_t": rdk.VerifyDesc, "rdk_multi_desc_t": rdk.MultiDesc, "rdk_kernel_desc_t": rdk.KernelDesc}
    for key, value in out.items():
        if "." in key:
            struct, field = key.split(".")
            assert getattr(mirrors[struct], field).offset == int(value), key
        else:
            assert ctypes.sizeof(mirrors[key]) == int(value), key


def test_bench_refuses_more_than_one_gpu():
    """Everything here runs on one GPU: asking bench.py for more ends at once with a message that says so."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and not r.stdout.strip()


def test_header_is_plain_c(tmp_path):
    """include/rdk.h on its own, as strict C99 and as C++: no torch or HIP types in the boundary."""
    import subprocess
    src = tmp_path / "only_header.c"
    src.write_text('#include "rdk.h"\nint main(void) { return 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, "-fsyntax-only", str(src)], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-I", inc, "-fsyntax-only", "-x", "c++", str(src)], check=True)
    text = open(os.path.join(inc, "rdk.h")).read()
    assert "torch" not in text and "hip/" not in text
