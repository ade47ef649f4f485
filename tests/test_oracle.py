"""Pins for the CPU oracle (oracle/conv_ref.c) against things that are not the oracle:
the paper's worked 5x5 example, brute-force lowering + library matmul (section 2.1 shapes,
both column orders of section 3.1), the 1x1 special case, delta filters, the closed-form
in-bounds tap count, the tap decomposition of section 3.2, and the stated output sizes."""
import os

import numpy as np
import pytest

import workloads
from oracle.conv_ref import conv_ref, out_dim

RNG = np.random.default_rng(12345)


def _rand(shape):
    return RNG.uniform(-1, 1, size=shape).astype(np.float32)


def lowered_matrix(x, R, S, stride, pad, dil, order):
    """Explicit im2col in fp64: (N*P*Q) x (R*S*C) matrix, columns in `order` ('rsc' or 'crs')."""
    N, H, W, C = x.shape
    P = (H + 2 * pad - dil * (R - 1) - 1) // stride + 1
    Q = (W + 2 * pad - dil * (S - 1) - 1) // stride + 1
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=np.float64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    cols = np.empty((N, P, Q, R, S, C), dtype=np.float64)
    for r in range(R):
        for s in range(S):
            cols[:, :, :, r, s, :] = xp[:, r * dil: r * dil + (P - 1) * stride + 1: stride,
                                        s * dil: s * dil + (Q - 1) * stride + 1: stride, :]
    if order == "rsc":
        return cols.reshape(N * P * Q, R * S * C), (N, P, Q)
    if order == "crs":
        return cols.transpose(0, 1, 2, 5, 3, 4).reshape(N * P * Q, C * R * S), (N, P, Q)
    raise ValueError(order)


def filter_matrix(w, order):
    K, R, S, C = w.shape
    w64 = w.astype(np.float64)
    if order == "rsc":
        return w64.reshape(K, R * S * C).T
    return w64.transpose(0, 3, 1, 2).reshape(K, C * R * S).T


SHAPES = [
    # N, H, W, C, K, R, S, stride, pad, dil
    (1, 5, 5, 8, 4, 3, 3, 1, 0, 1),
    (1, 5, 5, 8, 4, 3, 3, 2, 0, 1),
    (2, 7, 6, 3, 5, 3, 2, 1, 1, 1),
    (2, 9, 8, 4, 3, 3, 3, 2, 1, 1),
    (1, 11, 10, 5, 2, 3, 3, 1, 2, 2),
    (2, 12, 13, 2, 3, 7, 7, 2, 3, 1),
    (1, 6, 7, 6, 7, 1, 1, 2, 0, 1),
    (1, 9, 9, 2, 2, 3, 3, 3, 1, 2),
    (3, 4, 4, 1, 1, 2, 3, 1, 2, 1),
    (1, 8, 8, 16, 16, 3, 3, 1, 1, 1),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("order", ["rsc", "crs"])
def test_brute_force_lowering_times_matmul(shape, order):
    """Section 2.1: conv == lowered (P*Q x R*S*C) matrix times (C*R*S x K) filter matrix.
    Section 3.1: any column order gives the same product if the filter rows follow it."""
    N, H, W, C, K, R, S, st, pad, dil = shape
    x, w = _rand((N, H, W, C)), _rand((K, R, S, C))
    A, (n, p, q) = lowered_matrix(x, R, S, st, pad, dil, order)
    B = filter_matrix(w, order)
    assert A.shape[1] == R * S * C and B.shape == (C * R * S, K)
    want = (A @ B).reshape(n, p, q, K)
    got = conv_ref(x, w, st, pad, dil)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_1x1_stride1_is_plain_matmul():
    N, H, W, C, K = 2, 5, 7, 13, 9
    x, w = _rand((N, H, W, C)), _rand((K, 1, 1, C))
    want = x.reshape(-1, C).astype(np.float64) @ w.reshape(K, C).astype(np.float64).T
    got = conv_ref(x, w, 1, 0, 1)
    np.testing.assert_allclose(got.reshape(-1, K), want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("st,pad,dil", [(1, 0, 1), (1, 1, 1), (2, 1, 1), (1, 2, 2), (2, 3, 1), (3, 2, 2)])
def test_delta_filter_reproduces_shifted_input(st, pad, dil):
    """w[k,r0,s0,c] = [k == c] picks x[n, p*st + r0*dil - pad, q*st + s0*dil - pad, k], or 0
    outside the map.  Pins the spatial indexing, the absence of a filter flip and the padding."""
    N, H, W, C, R, S = 2, 9, 10, 4, 3, 3
    x = _rand((N, H, W, C))
    P = (H + 2 * pad - dil * (R - 1) - 1) // st + 1
    Q = (W + 2 * pad - dil * (S - 1) - 1) // st + 1
    for r0 in range(R):
        for s0 in range(S):
            w = np.zeros((C, R, S, C), dtype=np.float32)
            for c in range(C):
                w[c, r0, s0, c] = 1.0
            got = conv_ref(x, w, st, pad, dil)
            want = np.zeros((N, P, Q, C))
            for p in range(P):
                for q in range(Q):
                    h, ww = p * st + r0 * dil - pad, q * st + s0 * dil - pad
                    if 0 <= h < H and 0 <= ww < W:
                        want[:, p, q, :] = x[:, h, ww, :]
            assert np.array_equal(got, want)


def _in_bounds(P, size, filt, st, pad, dil):
    return np.array([sum(0 <= p * st + r * dil - pad < size for r in range(filt)) for p in range(P)])


# spatial geometry of the seven benchmark layers, with reduced N, C, K
GEOMS = {
    "cfg1": (8, 8, 3, 3, 1, 1, 1, 8, [2, 3, 3, 3, 3, 3, 3, 2]),
    "cfg2": (56, 56, 3, 3, 1, 1, 1, 56, None),
    "cfg3a": (56, 56, 3, 3, 2, 1, 1, 28, None),
    "cfg3b": (56, 56, 1, 1, 2, 0, 1, 28, None),
    "cfg4": (64, 64, 3, 3, 1, 2, 2, 64, None),
    "cfg5a": (224, 224, 7, 7, 2, 3, 1, 112, None),
    "cfg5b": (7, 7, 3, 3, 1, 1, 1, 7, [2, 3, 3, 3, 3, 3, 2]),
}


@pytest.mark.parametrize("name", list(GEOMS))
def test_all_ones_counts_in_bounds_taps(name):
    """x = 1, w = 1  =>  y[n,p,q,k] = C * rows_in(p) * cols_in(q): a closed form that checks
    padding, stride and dilation, and the output size each benchmark layer states."""
    H, W, R, S, st, pad, dil, PQ, rows_expected = GEOMS[name]
    L = workloads.LAYERS[name]
    assert (L.H, L.W, L.R, L.S, L.stride, L.pad, L.dilation) == (H, W, R, S, st, pad, dil)
    assert L.P == PQ and L.Q == PQ
    assert out_dim(H, R, st, pad, dil) == PQ and out_dim(W, S, st, pad, dil) == PQ
    C, K = 3, 2
    got = conv_ref(np.ones((1, H, W, C), np.float32), np.ones((K, R, S, C), np.float32), st, pad, dil)
    rows, cols = _in_bounds(PQ, H, R, st, pad, dil), _in_bounds(PQ, W, S, st, pad, dil)
    if rows_expected is not None:
        assert rows.tolist() == rows_expected
    want = C * rows[:, None] * cols[None, :]
    assert got.shape == (1, PQ, PQ, K)
    for k in range(K):
        assert np.array_equal(got[0, :, :, k], want)


def test_all_ones_edge_profiles():
    """Hand-derived edge profiles of the in-bounds row count for the benchmark geometries."""
    assert _in_bounds(28, 56, 3, 2, 1, 1).tolist() == [2] + [3] * 27            # 3x3 s2 p1
    assert _in_bounds(64, 64, 3, 1, 2, 2).tolist() == [2, 2] + [3] * 60 + [2, 2]  # 3x3 p2 d2
    assert _in_bounds(112, 224, 7, 2, 3, 1).tolist() == [4, 6] + [7] * 109 + [5]  # 7x7 s2 p3
    assert _in_bounds(28, 56, 1, 2, 0, 1).tolist() == [1] * 28


@pytest.mark.parametrize("shape", SHAPES)
def test_sum_of_decomposed_1x1_convs(shape):
    """Section 3.2: the layer is the sum over the R*S taps of a 1x1 conv on the shifted,
    strided input; order of accumulation is free."""
    N, H, W, C, K, R, S, st, pad, dil = shape
    x, w = _rand((N, H, W, C)), _rand((K, R, S, C))
    got = conv_ref(x, w, st, pad, dil)
    _, P, Q, _ = got.shape
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C))
    xp[:, pad:pad + H, pad:pad + W] = x
    acc = np.zeros_like(got)
    for r in reversed(range(R)):
        for s in range(S):
            sl = xp[:, r * dil: r * dil + (P - 1) * st + 1: st, s * dil: s * dil + (Q - 1) * st + 1: st, :]
            acc += sl @ w[:, r, s, :].astype(np.float64).T
    np.testing.assert_allclose(got, acc, rtol=0, atol=1e-12)


# ---- the paper's worked 5x5 example ---------------------------------------------------------

def _golden(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "paper_5x5_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = [t.strip() for t in line.split("=")]
            out[k] = v.split()
    return out


def _pos(label):
    return int(label[0]) - 1, "ABCDE".index(label[1])


def test_paper_window_read_order(golden_dir):
    """Section 3.1: window (0,0) reads 1A..3C, window (0,1) reads 1B..3D, taps row by row.
    A one-hot input at the i-th listed position times the filter w[r,s] = 1 + 3r + s must give
    i + 1 at that window (wrong order, a flip, or a transposed index gives another number)."""
    g = _golden(golden_dir)
    w = (1 + np.arange(9, dtype=np.float32)).reshape(1, 3, 3, 1)
    for key, (p, q) in (("window_stride1_p0_q0", (0, 0)), ("window_stride1_p0_q1", (0, 1))):
        seq = g[key]
        assert len(seq) == 9
        for i, label in enumerate(seq):
            x = np.zeros((1, 5, 5, 1), np.float32)
            x[0, _pos(label)[0], _pos(label)[1], 0] = 1.0
            y = conv_ref(x, w, 1, 0, 1)
            assert y.shape == (1, 3, 3, 1)
            assert y[0, p, q, 0] == i + 1


def test_paper_stride2_tap_footprints(golden_dir):
    """Section 3.2, Fig. 8a: at stride 2 tap <1,1> touches 1A 1C 3A 3C and tap <1,2> touches
    1B 1D 3B 3D.  With x[h,w] = 2^(5h+w) and a filter that is 1 at one tap, the sum of the
    outputs is the bit set of touched positions."""
    g = _golden(golden_dir)
    x = (2.0 ** np.arange(25)).astype(np.float32).reshape(1, 5, 5, 1)
    for key, (r, s) in (("tap_stride2_r0_s0", (0, 0)), ("tap_stride2_r0_s1", (0, 1))):
        w = np.zeros((1, 3, 3, 1), np.float32)
        w[0, r, s, 0] = 1.0
        y = conv_ref(x, w, 2, 0, 1)
        assert y.size == int(g["outputs_stride2"][0])
        bits = int(y.sum())
        touched = {f"{h + 1}{'ABCDE'[c]}" for h in range(5) for c in range(5) if bits >> (5 * h + c) & 1}
        assert touched == set(g[key])
        # and the output pixels come in row-major (p, q) order
        want = [x[0, _pos(l)[0], _pos(l)[1], 0] for l in g[key]]
        assert y.reshape(-1).tolist() == want


def test_paper_output_counts(golden_dir):
    g = _golden(golden_dir)
    x = np.ones((1, 5, 5, 8), np.float32)
    w = np.ones((2, 3, 3, 8), np.float32)
    assert conv_ref(x, w, 1, 0, 1).shape[1:3] == (3, 3) and 9 == int(g["outputs_stride1"][0])
    assert conv_ref(x, w, 2, 0, 1).shape[1:3] == (2, 2) and 4 == int(g["outputs_stride2"][0])


def test_lowered_matrix_memory_ratio():
    """Section 2.2 ("Memory Overhead"): the lowered matrix is at most R*S times the input.
    Closed form M*C*R*S / (N*H*W*C) for the benchmark layers."""
    want = {"cfg2": 9.0, "cfg3a": 2.25, "cfg3b": 0.25, "cfg4": 9.0, "cfg5a": 12.25, "cfg5b": 9.0, "cfg1": 9.0}
    for name, ratio in want.items():
        L = workloads.LAYERS[name]
        got = L.M * L.k_gemm / (L.N * L.H * L.W * L.C)
        assert got == ratio and got <= L.R * L.S


def test_rejects_bad_arguments():
    x, w = np.ones((1, 2, 2, 1), np.float32), np.ones((1, 3, 3, 1), np.float32)
    with pytest.raises(ValueError):
        conv_ref(x, w, 1, 0, 1)          # filter larger than the map: empty output
    with pytest.raises(ValueError):
        conv_ref(x, np.ones((1, 1, 1, 2), np.float32))  # channel mismatch


# ---- the shared input generator ------------------------------------------------------------

def test_round_to_grid_matches_torch_casts():
    torch = pytest.importorskip("torch")
    a = np.concatenate([_rand(4096) * 3, np.float32([0, -0.0, 1, 1 + 2 ** -8, 1 + 3 * 2 ** -8, 65504, 1e-8])])
    for name, tdt in (("bf16", torch.bfloat16), ("f16", torch.float16)):
        want = torch.from_numpy(a).to(tdt).to(torch.float32).numpy()
        assert np.array_equal(workloads.round_to_grid(a, name), want)
    assert np.array_equal(workloads.round_to_grid(a, "f32"), a)


def test_make_inputs_seeded_and_scaled():
    L = workloads.LAYERS["cfg1"]
    x1, w1 = workloads.make_inputs(L)
    x2, w2 = workloads.make_inputs(L)
    assert np.array_equal(x1, x2) and np.array_equal(w1, w2)
    assert x1.shape == (1, 8, 8, 16) and w1.shape == (16, 3, 3, 16)
    assert abs(x1).max() <= 1 and abs(w1).max() <= 1 / np.sqrt(16 * 9) + 1e-7
    S = workloads.small_layer("stem", 1, 9, 9, 4, 2, 7, 7, 2, 3)
    S = workloads.ConvLayer(**{**S.__dict__, "c_real": 3})
    x, w = workloads.make_inputs(S)
    assert not x[..., 3].any() and not w[..., 3].any() and x[..., :3].any()
