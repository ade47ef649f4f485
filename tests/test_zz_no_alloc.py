"""The allocation-free explicit entry point (for callers that cannot call hipMalloc) against the
entry point it is a variant of, iconv_fwd_explicit, through the C ABI: same kernels, so the outputs
must be bit-equal; also checked against the oracle.  Two calls in a row share the library's one
device buffer, the second on a smaller layer."""
import numpy as np
import pytest

import workloads
from oracle.conv_ref import conv_ref

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2110_03901_amd import binding
    return binding


def run_pair(B, L, code):
    x, w = workloads.make_inputs(L)
    xd, wd = B.to_device(x, code), B.to_device(w, code)
    nbytes = B.iconv_workspace_bytes(B.ALGO_EXPLICIT, *L.shape_args(), code)
    assert 0 < nbytes <= B.NOALLOC_WORKSPACE_BYTES
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    want = B.empty_output(L.N, L.P, L.Q, L.K, code)
    want.fill_(float("nan"))
    B.iconv_fwd_explicit(xd, wd, want, ws, nbytes, *L.shape_args(), code)
    got = B.empty_output(L.N, L.P, L.Q, L.K, code)
    got.fill_(float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.iconv_fwd_explicit_noalloc(xd, wd, got, *L.shape_args(), code)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.isfinite(got.float()).all(), "some output was not written"
    assert torch.equal(got, want), f"{L.name}: differs from iconv_fwd_explicit"
    ref = conv_ref(x, w, L.stride, L.pad, L.dilation)
    err = np.abs(got.float().cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max()
    print(f"{L.name}: lowered matrix {nbytes} B, rel_err vs oracle {err:.3e}", flush=True)
    assert err <= (1e-4 if code in (1, 2) else 2.0 ** -8 * 1.01)


def test_two_calls_in_a_row_second_smaller(B):
    big = workloads.small_layer("na_big", 4, 56, 56, 64, 64, 3, 3, 1, 1, 1, seed_id=990)        # 14.45 MB lowered
    small = workloads.small_layer("na_small", 2, 15, 17, 32, 40, 3, 3, 2, 1, 1, seed_id=991)    # strided, ragged K
    run_pair(B, big, 1)
    run_pair(B, small, 1)
    run_pair(B, workloads.small_layer("na_f16", 1, 20, 20, 16, 24, 5, 3, 1, 2, 1, dtype="f16", seed_id=992), 4)
    run_pair(B, big, 1)                                                                         # and the large one again


def test_sizes_beyond_the_buffer_are_rejected(B):
    L = workloads.LAYERS["cfg2"]                   # 115.6 MB lowered
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    assert B.iconv_workspace_bytes(B.ALGO_EXPLICIT, *L.shape_args(), 1) > B.NOALLOC_WORKSPACE_BYTES
    assert B.iconv_fwd_explicit_noalloc_raw(t, t, t, *L.shape_args(), 1) == -5
    assert B.iconv_fwd_explicit_noalloc_raw(t, t, None, 1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 1) == -1
    assert B.iconv_fwd_explicit_noalloc_raw(t, t, t, 1, 8, 8, 16, 16, 3, 3, 1, 1, 1, 9) == -3
