"""CPU sanitizer leg: the oracle (gcc) and the host half of the C ABI (hipcc's host pass) built with
AddressSanitizer and UndefinedBehaviorSanitizer, then driven through the oracle's pins and the ABI's
argument checks in a child process that preloads the sanitizer runtime.  Any report makes the child
exit non-zero.  No GPU is involved: device code is compiled as usual and never runs here."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUILD = os.path.join(ROOT, "_build", "sanitize")


def run_child(code, preload, extra_env):
    env = dict(os.environ)
    env.update(extra_env)
    env["LD_PRELOAD"] = preload + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # python itself leaks by design; a real error still aborts (exit code 1 via halt_on_error)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, f"exit {r.returncode}\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    return r.stdout


def test_oracle_under_address_and_ub_sanitizers():
    os.makedirs(BUILD, exist_ok=True)
    lib = os.path.join(BUILD, "libconv_ref_asan.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", lib, os.path.join(ROOT, "oracle", "conv_ref.c")])
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    code = r'''
import numpy as np
from oracle.conv_ref import conv_ref, out_dim
rng = np.random.default_rng(5)
# shapes with every kind of border: padding wider than the filter, dilation, stride, P or Q = 1, single pixel
cases = [(1, 8, 8, 16, 16, 3, 3, 1, 1, 1), (2, 6, 6, 4, 3, 3, 3, 1, 4, 1), (2, 20, 19, 5, 7, 3, 3, 3, 2, 2), (1, 40, 3, 6, 8, 3, 3, 1, 0, 1),
         (1, 1, 1, 8, 1, 1, 1, 1, 0, 1), (3, 9, 7, 3, 5, 5, 3, 2, 2, 1), (1, 12, 12, 2, 2, 7, 7, 2, 3, 1)]
for N, H, W, C, K, R, S, st, pad, dil in cases:
    x = rng.uniform(-1, 1, (N, H, W, C)).astype(np.float32)
    w = rng.uniform(-1, 1, (K, R, S, C)).astype(np.float32)
    y = conv_ref(x, w, st, pad, dil)
    P, Q = out_dim(H, R, st, pad, dil), out_dim(W, S, st, pad, dil)
    assert y.shape == (N, P, Q, K)
    # brute-force lowering x matmul (section 2.1): the same pin as tests/test_oracle.py, here under the sanitizers
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C)); xp[:, pad:pad + H, pad:pad + W] = x
    low = np.stack([xp[:, r * dil: r * dil + (P - 1) * st + 1: st, s * dil: s * dil + (Q - 1) * st + 1: st]
                    for r in range(R) for s in range(S)], axis=3).reshape(N * P * Q, R * S * C)
    want = (low @ w.reshape(K, -1).astype(np.float64).T).reshape(N, P, Q, K)
    assert np.abs(y - want).max() < 1e-12
try:
    conv_ref(np.zeros((1, 2, 2, 1), np.float32), np.zeros((1, 3, 3, 1), np.float32))   # empty output: rejected, not computed
    raise SystemExit("empty output accepted")
except ValueError:
    pass
print("oracle ok")
'''
    out = run_child(code, asan, {"CONV_REF_LIB": lib})
    assert "oracle ok" in out


def test_abi_argument_checks_under_address_and_ub_sanitizers():
    hipcc = "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2110_03901_amd import build as pkg_build
    main_lib = pkg_build.LIB
    if not os.path.exists(main_lib):
        pkg_build.build_library(verbose=False)
    os.makedirs(BUILD, exist_ok=True)
    csrc = pkg_build.CSRC
    api_o = os.path.join(BUILD, "iconv_api_asan.o")
    flags = [f for f in pkg_build.HIPCC_FLAGS if f != "-O3"]
    # (sanitizers on the host pass only: each -fsanitize= directly after -Xarch_host)
    subprocess.check_call([hipcc, "-O1", "-g", *flags, "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                           "-Xarch_host", "-fno-sanitize-recover=all", "-c", os.path.join(csrc, "iconv_api.hip"), "-o", api_o],
                          stderr=subprocess.DEVNULL)
    objs = [os.path.join(csrc, src.replace(".hip", ".o")) for src in pkg_build.SOURCES if src != "iconv_api.hip"]
    lib = os.path.join(BUILD, "libiconv_asan.so")
    rt = subprocess.check_output(["/opt/rocm/lib/llvm/bin/clang", "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                           "-shared-libsan", "-o", lib, api_o, *objs], stderr=subprocess.DEVNULL)
    code = r'''
import ctypes, os
lib = ctypes.CDLL(os.environ["ICONV_ASAN_LIB"])
i, p, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
lib.iconv_fwd.argtypes = [p] * 3 + [i] * 11 + [p]
lib.iconv_fwd_ex.argtypes = [p] * 3 + [i] * 13 + [p]
lib.iconv_fwd_explicit.argtypes = [p] * 4 + [sz] + [i] * 11 + [p]
lib.iconv_fwd_explicit_noalloc.argtypes = [p] * 3 + [i] * 11 + [p]
lib.iconv_workspace_bytes.restype = sz
lib.iconv_kernel_for.restype = ctypes.c_char_p
lib.iconv_status_string.restype = ctypes.c_char_p
ok = (1, 8, 8, 16, 16, 3, 3, 1, 1, 1)
a = 4096
P, Q = i(), i()
assert lib.iconv_out_shape(56, 56, 3, 3, 2, 1, 1, ctypes.byref(P), ctypes.byref(Q)) == 0 and (P.value, Q.value) == (28, 28)
assert lib.iconv_out_shape(2, 2, 3, 3, 1, 0, 1, ctypes.byref(P), ctypes.byref(Q)) == -2
assert lib.iconv_fwd(None, a, a, *ok, 1, None) == -1
assert lib.iconv_fwd(a, a, a, 1, 8, 8, 0, 16, 3, 3, 1, 1, 1, 1, None) == -2
assert lib.iconv_fwd(a, a, a, *ok, 9, None) == -3
assert lib.iconv_fwd(a, a, a, 4, 32768, 32768, 16, 16, 3, 3, 1, 1, 1, 1, None) == -3
assert lib.iconv_fwd(a, a, a, 2147483647, 2147483647, 2147483647, 2147483647, 2147483647, 7, 7, 1, 2147483647, 1, 1, None) == -3
assert lib.iconv_fwd(a + 8, a, a, *ok, 1, None) == -4
assert lib.iconv_fwd_ex(a, a, a, *ok, 1, 999, 0, None) == -3
assert lib.iconv_fwd_ex(a, a, a, *ok, 1, -1, -5, None) == -3
assert lib.iconv_fwd_explicit(a, a, a, a, 16, *ok, 1, None) == -5
assert lib.iconv_fwd_explicit_noalloc(a, a, a, 32, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1, None) == -5
assert lib.iconv_workspace_bytes(1, 32, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1) == 100352 * 576 * 2
assert lib.iconv_workspace_bytes(1, 1, 2, 2, 1, 1, 3, 3, 1, 0, 1, 1) == 0
for args in [(32, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1), (64, 7, 7, 512, 512, 3, 3, 1, 1, 1, 1), (64, 224, 224, 4, 64, 7, 7, 2, 3, 1, 1),
             (3, 17, 19, 8, 8, 1, 1, 1, 0, 1, 2), (2147483647, 1, 1, 8, 8, 1, 1, 1, 0, 1, 1), (1, 1, 1, 8, 1, 1, 1, 1, 2147483647, 1, 1),
             (32, 56, 56, 256, 512, 1, 1, 2, 0, 1, 1), (2147483647, 1, 1, 64, 8, 1, 1, 1, 0, 1, 1), (1, 16383, 16383, 64, 4, 1, 1, 1, 0, 1, 1),
             (4, 16384, 8, 128, 2147483644, 1, 1, 1, 0, 1, 1)]:
    lib.iconv_kernel_for(*args)
for v in range(-2, lib.iconv_num_variants() + 2):
    lib.iconv_variant_accepts(v, 2, 24, 24, 64, 64, 3, 3, 1, 1, 1, 1)
assert len({lib.iconv_status_string(c) for c in range(0, -8, -1)}) == 8
print("abi ok")
'''
    out = run_child(code, rt, {"ICONV_ASAN_LIB": lib})
    assert "abi ok" in out
