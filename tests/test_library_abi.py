"""Host-only checks of the HIP library: it loads, exports every symbol the header declares,
and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2603_04135_amd as P
    if not os.path.exists(P.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return P.load()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dppo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dppo_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2603_04135_amd.binding import EXPORTS
    declared = _declared_symbols()
    assert declared, "no declarations found in include/dppo.h"
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(EXPORTS) == declared


def test_status_strings(lib):
    assert lib.dppo_status_str(0) == b"ok"
    assert lib.dppo_status_str(3) and lib.dppo_status_str(99) == b"unknown status"
    assert lib.dppo_last_error() is not None


def test_host_side_validation_launches_nothing(lib):
    from paper_2603_04135_amd.binding import HeadShape, LossParams, PackParams, SelectParams
    one = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    sp = SelectParams(4, 4, 1.0, 0.5, 1e-6, 1, 0.5, 0, 1)       # r_q outside [0,1)
    assert lib.dppo_select(ctypes.byref(sp), *([one] * 14), None) == 1
    assert b"[0,1)" in lib.dppo_last_error()
    sp = SelectParams(4, 1, 0.5, 0.5, 1e-6, 1, 0.5, 0, 1)       # sample std of one completion
    assert lib.dppo_select(ctypes.byref(sp), *([one] * 14), None) == 2
    sp = SelectParams(4, 4, 0.5, 0.5, 1e-6, 1, 0.5, 0, 1)
    assert lib.dppo_select(ctypes.byref(sp), None, *([one] * 13), None) == 1
    sp = SelectParams(4, 4, 0.5, 0.5, 0.0, 1, 0.5, 0, 1)        # adv_eps = 0: a constant group would divide 0 by 0
    assert lib.dppo_select(ctypes.byref(sp), *([one] * 14), None) == 1
    pp = PackParams(0, 16, 4, 0)
    assert lib.dppo_pack(ctypes.byref(pp), *([one] * 8), 10, one, None) == 2
    pp = PackParams(4, 16, 0, 0)
    assert lib.dppo_pack(ctypes.byref(pp), *([one] * 8), 10, one, None) == 1
    pp = PackParams(4, 16, 4, 7)                          # unknown policy
    assert lib.dppo_pack(ctypes.byref(pp), *([one] * 8), 10, one, None) == 1
    pp = PackParams(4, 1, 4, 0)                           # capacity below a 1+1 token item
    assert lib.dppo_pack(ctypes.byref(pp), *([one] * 8), 10, one, None) == 3
    hs = HeadShape(100, 50, 72, 1000, 1)                  # bf16 needs D % 64 == 0
    assert lib.dppo_token_logprob(ctypes.byref(hs), *([one] * 8), 1 << 20, None) == 5
    assert lib.dppo_workspace_bytes(ctypes.byref(hs), 1) == 0
    hs = HeadShape(100, 200, 64, 1000, 1)                 # N > T
    assert lib.dppo_token_logprob(ctypes.byref(hs), *([one] * 8), 1 << 20, None) == 2
    hs = HeadShape(100, 50, 64, 1000, 1)
    lp = LossParams(0.2, 0.2, 0.04, 0, 0)
    assert lib.dppo_loss_fwd_bwd(ctypes.byref(hs), ctypes.byref(lp), 3, *([one] * 16), one, 1024, None) == 4
    assert lib.dppo_token_logprob(ctypes.byref(hs), *([one] * 7), None, 1 << 20, None) == 4
    lp = LossParams(0.2, 0.2, 0.04, 0, 0, 2, 0)          # unknown ratio level
    assert lib.dppo_loss_fwd_bwd(ctypes.byref(hs), ctypes.byref(lp), 3, *([one] * 16), one, 1 << 30, None) == 1
    assert lib.dppo_token_norm_coef(0, 4, one, one, one, None) == 2
    assert lib.dppo_variance_terms(4, 0, one, one, one, one, one, None) == 2
    assert lib.dppo_variance_terms(4, 4, one, None, one, one, one, None) == 1


def test_workspace_sizes(lib):
    from paper_2603_04135_amd.binding import HeadShape
    hs = HeadShape(370000, 310000, 2560, 151936, 1)
    rec = lib.dppo_workspace_bytes(ctypes.byref(hs), 1)
    mn = lib.dppo_workspace_min_bytes(ctypes.byref(hs), 1)
    fwd = lib.dppo_workspace_bytes(ctypes.byref(hs), 0)
    assert 0 < fwd < mn < rec < 40 * 2**30


def test_validation_paths_under_host_sanitizers(tmp_path):
    """Builds the library's host code with AddressSanitizer and UndefinedBehaviorSanitizer (host side only; the
    device code is compiled as always) together with tests/abi_host_check.c, a plain-C driver that walks every
    entry point's argument validation and the workspace arithmetic, and runs it: no report, exit status 0."""
    import shutil
    import subprocess
    from concurrent.futures import ThreadPoolExecutor

    import torch
    from paper_2603_04135_amd import build as B

    hipcc = B._hipcc()
    clang = shutil.which("amdclang") or "/opt/rocm/llvm/bin/clang"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]
    jobs, objs = [], []
    for src in B.SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        objs.append(obj)
        jobs.append([hipcc, *B.COMMON_FLAGS, *B.PER_FILE_FLAGS.get(src, []), *san, "-c", os.path.join(B.CSRC, src), "-o", obj])
    chk = str(tmp_path / "abi_host_check.o")
    jobs.append([clang, "-std=c11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-g", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=undefined", "-I", B.INCLUDE, "-c", os.path.join(ROOT, "tests", "abi_host_check.c"), "-o", chk])
    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(B._run, jobs))
    exe = str(tmp_path / "abi_host_check")
    B._run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", *objs, chk, "-o", exe])
    symbols = subprocess.run(["nm", exe], stdout=subprocess.PIPE, text=True).stdout
    assert "__asan_report" in symbols and "__ubsan_handle" in symbols, "the sanitizers are not linked in"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               DPPO_ABI_CHECK_NO_GPU="0" if torch.cuda.is_available() else "1")
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    assert proc.returncode == 0 and "abi_host_check: ok" in proc.stdout, proc.stdout + proc.stderr
    assert "runtime error" not in proc.stderr and "AddressSanitizer" not in proc.stderr, proc.stderr
