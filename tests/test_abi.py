"""CPU-side checks of the boundary: the library loads, exports every symbol the two headers
declare (include/iconv.h: the convolution contract; include/iconv_bench.h: test and measurement
entry points), and its host-only entry points (shape, workspace size, status strings, argument
validation that returns before any launch) behave as the headers state."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2110_03901_amd", "libiconv_mi355.so")
HEADER = os.path.join(ROOT, "include", "iconv.h")
HEADER_BENCH = os.path.join(ROOT, "include", "iconv_bench.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2110_03901_amd.build import build_library
        build_library(verbose=False)
    return ctypes.CDLL(LIB)


def declared_functions(header):
    text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(iconv_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = declared_functions(HEADER)
    assert {"iconv_fwd", "iconv_out_shape", "iconv_workspace_bytes", "iconv_fwd_explicit", "iconv_status_string"} <= set(names)
    bench = declared_functions(HEADER_BENCH)
    assert {"iconv_fwd_ex", "iconv_num_variants", "iconv_variant_name", "iconv_variant_accepts", "iconv_probe_copy",
            "iconv_probe_copy_wt", "iconv_probe_mfma", "iconv_probe_lds", "iconv_lds_swizzle", "iconv_lds_stage_offset"} == set(bench)
    for n in names + bench:
        assert hasattr(lib, n), f"{n} is declared in a header but not exported"


def test_contract_header_declares_no_switches():
    """iconv.h is the convolution contract: no process-wide override and no measurement helper is
    declared there, and the binding lists the same symbols as the headers."""
    names = set(declared_functions(HEADER))
    assert not any(n.startswith(("iconv_set_", "iconv_probe_")) for n in names)
    src = open(os.path.join(ROOT, "paper_2110_03901_amd", "binding.py")).read()
    listed = set(re.findall(r'"(iconv_[a-z0-9_]+)"', src.split("EXPORTS =")[1].split("\n\n")[0]))
    assert "iconv_fwd_ex" in listed
    assert listed == names | set(declared_functions(HEADER_BENCH))


def test_out_shape(lib):
    P, Q = ctypes.c_int(), ctypes.c_int()
    cases = [((56, 56, 3, 3, 1, 1, 1), (56, 56)), ((56, 56, 3, 3, 2, 1, 1), (28, 28)),
             ((56, 56, 1, 1, 2, 0, 1), (28, 28)), ((64, 64, 3, 3, 1, 2, 2), (64, 64)),
             ((224, 224, 7, 7, 2, 3, 1), (112, 112)), ((7, 7, 3, 3, 1, 1, 1), (7, 7)),
             ((5, 5, 3, 3, 1, 0, 1), (3, 3)), ((5, 5, 3, 3, 2, 0, 1), (2, 2)), ((9, 4, 3, 2, 3, 1, 2), (3, 2))]
    for args, want in cases:
        assert lib.iconv_out_shape(*args, ctypes.byref(P), ctypes.byref(Q)) == 0
        assert (P.value, Q.value) == want
    assert lib.iconv_out_shape(2, 2, 3, 3, 1, 0, 1, ctypes.byref(P), ctypes.byref(Q)) == -2
    assert lib.iconv_out_shape(8, 8, 3, 3, 0, 0, 1, ctypes.byref(P), ctypes.byref(Q)) == -2
    assert lib.iconv_out_shape(8, 8, 3, 3, 1, 0, 1, None, ctypes.byref(Q)) == -1


def test_workspace_bytes(lib):
    lib.iconv_workspace_bytes.restype = ctypes.c_size_t
    import workloads
    for L in workloads.LAYERS.values():
        code = 0 if L.dtype == "f32" else 1
        assert lib.iconv_workspace_bytes(0, *L.shape_args(), code) == 0          # implicit: none
        want = L.M * L.k_gemm * L.elt_bytes()                                    # the lowered matrix of section 2.1
        if code != 0 and L.k_gemm % 8:
            # 16-bit rows padded to a multiple of 8 elements, total rounded to 16 bytes, + the filter matrix at that pitch
            pitch = (L.k_gemm + 7) // 8 * 8
            want = (L.M * pitch * 2 + 15) // 16 * 16 + L.K * pitch * 2
            assert L.name == "cfg5a" and pitch == 200
        assert lib.iconv_workspace_bytes(1, *L.shape_args(), code) == want
    assert lib.iconv_workspace_bytes(1, 1, 2, 2, 1, 1, 3, 3, 1, 0, 1, 1) == 0    # invalid shape


def test_validation_happens_before_any_launch(lib):
    f = lib.iconv_fwd
    f.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 11 + [ctypes.c_void_p]
    ok = (1, 8, 8, 16, 16, 3, 3, 1, 1, 1)
    a = 4096  # a non-null, 16-byte aligned fake address; never dereferenced on these paths
    assert f(None, a, a, *ok, 1, None) == -1
    assert f(a, a, None, *ok, 1, None) == -1
    assert f(a, a, a, 1, 8, 8, 0, 16, 3, 3, 1, 1, 1, 1, None) == -2
    assert f(a, a, a, 1, 2, 2, 16, 16, 3, 3, 1, 0, 1, 1, None) == -2     # empty output
    assert f(a, a, a, 1, 8, 8, 16, 16, 3, 3, 1, -1, 1, 1, None) == -2
    assert f(a, a, a, *ok, 9, None) == -3                                # unknown dtype
    assert f(a, a, a, 4, 32768, 32768, 16, 16, 3, 3, 1, 1, 1, 1, None) == -3  # >= 2^31 elements
    assert f(a + 8, a, a, *ok, 1, None) == -4
    e = lib.iconv_fwd_explicit
    e.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_size_t] + [ctypes.c_int] * 11 + [ctypes.c_void_p]
    assert e(a, a, a, a, 16, *ok, 1, None) == -5
    assert e(a, a, a, None, 1 << 30, *ok, 1, None) == -5


def test_status_strings_and_variants(lib):
    lib.iconv_status_string.restype = ctypes.c_char_p
    seen = {lib.iconv_status_string(c) for c in range(0, -7, -1)}
    assert len(seen) == 7 and lib.iconv_status_string(0) == b"ok"
    lib.iconv_variant_name.restype = ctypes.c_char_p
    n = lib.iconv_num_variants()
    assert n >= 1 and len({lib.iconv_variant_name(i) for i in range(n)}) == n
    assert lib.iconv_variant_name(n) == b"auto" and lib.iconv_variant_name(-1) == b"auto"


def test_extended_call_validates_its_overrides(lib):
    f = lib.iconv_fwd_ex
    f.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 13 + [ctypes.c_void_p]
    ok = (1, 8, 8, 16, 16, 3, 3, 1, 1, 1)
    a = 4096  # fake aligned address, never dereferenced on these paths
    n = lib.iconv_num_variants()
    assert f(a, a, a, *ok, 1, n, 0, None) == -3          # no such kernel-table entry
    assert f(a, a, a, *ok, 1, -2, 0, None) == -3
    assert f(a, a, a, *ok, 1, -1, -1, None) == -3        # negative workgroup cap
    assert f(None, a, a, *ok, 1, -1, 0, None) == -1
    assert f(a, a, a, 1, 2, 2, 16, 16, 3, 3, 1, 0, 1, 1, -1, 0, None) == -2
    assert f(a + 4, a, a, *ok, 1, 0, 0, None) == -4


def kernel_for(lib, *args):
    lib.iconv_kernel_for.restype = ctypes.c_char_p
    lib.iconv_kernel_for.argtypes = [ctypes.c_int] * 11
    r = lib.iconv_kernel_for(*args)
    return None if r is None else r.decode()


def test_kernel_choice_follows_the_layer_class(lib):
    """iconv_kernel_for (host logic; 256 compute units are assumed without a device): each class of layer gets the
    kernel family built for it, every answer is a kernel-table name or "direct", invalid arguments give NULL."""
    lib.iconv_variant_name.restype = ctypes.c_char_p
    table = {lib.iconv_variant_name(i).decode() for i in range(lib.iconv_num_variants())}
    bf16 = 1
    # the benchmark layers: resident filters (s..., t...: phased by filter row; r...: by channel slice), per-tap
    # direct-to-LDS (d...), patch reuse (p...), merged taps
    assert kernel_for(lib, 32, 56, 56, 64, 64, 3, 3, 1, 1, 1, bf16).startswith("s448")          # 224 blocks: one round, all waves compute
    assert kernel_for(lib, 64, 56, 56, 64, 64, 3, 3, 1, 1, 1, bf16).startswith("t448")          # 448 blocks: persistent, loader waves
    assert kernel_for(lib, 32, 56, 56, 96, 64, 1, 1, 1, 0, 1, bf16).startswith("r")            # 96 channels: channel slices
    assert kernel_for(lib, 32, 56, 56, 128, 128, 3, 3, 2, 1, 1, bf16).startswith("d128x128")
    assert kernel_for(lib, 32, 56, 56, 256, 512, 1, 1, 2, 0, 1, bf16) == "a128x32_2x4+4+4"        # 1x1: pixels resident, store waves
    assert kernel_for(lib, 8, 64, 64, 256, 256, 3, 3, 1, 2, 2, bf16).startswith("p256x128")
    assert kernel_for(lib, 64, 7, 7, 512, 512, 3, 3, 1, 1, 1, bf16) == "p64x128_c128_w32x64_s3_4x2+4"   # one round: K split over two waves
    assert kernel_for(lib, 96, 7, 7, 512, 512, 3, 3, 1, 1, 1, bf16) == "p64x128_c128_w32x64_s3_4+4"    # 384 tiles: more than one round
    assert kernel_for(lib, 64, 224, 224, 4, 64, 7, 7, 2, 3, 1, bf16) == "stem_8+4"           # 12 blocks per compute unit: store waves
    assert kernel_for(lib, 8, 224, 224, 4, 64, 7, 7, 2, 3, 1, bf16) == "stem"                # 1.5 blocks per compute unit
    assert kernel_for(lib, 4, 224, 224, 4, 64, 7, 7, 2, 3, 1, bf16) == "stem_8+4"            # at most one block per compute unit
    assert kernel_for(lib, 64, 224, 224, 4, 62, 7, 7, 2, 3, 1, bf16) == "stem"               # K % 4 != 0
    assert kernel_for(lib, 1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 0) == "direct"            # fp32
    assert kernel_for(lib, 2, 8, 8, 20, 16, 3, 3, 1, 1, 1, bf16) == "direct"         # C % 8 != 0
    # tile size follows the tile count: the same layers at other batch sizes
    assert kernel_for(lib, 8, 56, 56, 64, 64, 3, 3, 1, 1, 1, bf16).startswith("p128x64")      # 196 tiles of 128 pixels
    assert kernel_for(lib, 16, 56, 56, 64, 64, 3, 3, 1, 1, 1, bf16).startswith("p256x64")     # 112 resident blocks: too few
    assert kernel_for(lib, 20, 56, 56, 64, 64, 3, 3, 1, 1, 1, bf16).startswith("s")           # patch tiles need two rounds
    assert kernel_for(lib, 64, 56, 56, 128, 128, 3, 3, 2, 1, 1, bf16).startswith("d256x128")  # 392 tiles of 128x128
    assert kernel_for(lib, 32, 56, 56, 256, 128, 1, 1, 1, 0, 1, bf16).startswith("d256x128")  # K = 128: no 256-wide tile;
    #   several rounds of workgroups that fill a compute unit's LDS and write four tiles each: not for the pixel-resident
    #   kernels, nor are 49 pixels per workgroup; with 16 tiles to write, or 74 pixels, the form with store waves
    assert kernel_for(lib, 64, 56, 56, 256, 512, 1, 1, 2, 0, 1, bf16) == "a128x32_2x4+4+4"
    assert kernel_for(lib, 64, 56, 56, 256, 256, 1, 1, 2, 0, 1, bf16).startswith("d256x256")
    assert kernel_for(lib, 16, 56, 56, 256, 512, 1, 1, 2, 0, 1, bf16).startswith("d")
    assert kernel_for(lib, 24, 56, 56, 256, 512, 1, 1, 2, 0, 1, bf16) == "a128x32_2x4+4+4"
    assert kernel_for(lib, 32, 56, 56, 64, 256, 1, 1, 1, 0, 1, bf16) == "a128x32_2x4+8"       # 64 channels: several per compute unit
    assert kernel_for(lib, 32, 28, 28, 128, 1024, 1, 1, 1, 0, 1, bf16) == "a128x32_2x4+4+4"   # 128 channels, 32 filter tiles per workgroup: store waves
    assert kernel_for(lib, 32, 28, 28, 128, 512, 1, 1, 1, 0, 1, bf16) == "a128x32_2x4+8"      # ... 16 tiles: two workgroups per compute unit overlap as well
    assert kernel_for(lib, 24, 28, 28, 128, 256, 1, 1, 1, 0, 1, bf16) == "a128x32_2x4+4+4"    # 74 pixels per workgroup
    assert kernel_for(lib, 32, 56, 56, 128, 128, 1, 1, 1, 0, 1, bf16) == "a128x32_2x4+8"      # four tiles: the compute waves store
    assert kernel_for(lib, 32, 7, 7, 2048, 512, 1, 1, 1, 0, 1, bf16).startswith("d64x64")     # 1568 output pixels
    for args in [(3, 17, 19, 8, 8, 1, 1, 1, 0, 1, 2), (5, 9, 33, 48, 24, 5, 3, 2, 2, 1, 3), (1, 1, 1, 8, 1, 1, 1, 1, 0, 1, 4),
                 (2, 40, 40, 96, 200, 3, 3, 1, 4, 4, bf16), (7, 12, 12, 64, 64, 3, 3, 1, 1, 1, bf16)]:
        name = kernel_for(lib, *args)
        assert name in table or name == "direct", (args, name)
    # what iconv_fwd rejects
    assert kernel_for(lib, 0, 8, 8, 16, 16, 3, 3, 1, 1, 1, bf16) is None             # shape
    assert kernel_for(lib, 1, 2, 2, 16, 16, 3, 3, 1, 0, 1, bf16) is None             # empty output
    assert kernel_for(lib, 1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 9) is None                # dtype
    assert kernel_for(lib, 4096, 1024, 1024, 8, 8, 1, 1, 1, 0, 1, bf16) is None      # 2^31 elements or more
