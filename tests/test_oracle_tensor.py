"""Pins for the fp64 tensor oracle (CPU only).

Each test ties the oracle to something other than itself: independently written
index arithmetic on tiny integer inputs (exact), closed forms, special cases that
reduce to another pinned operator, and library routines in float64.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import tensor as T

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _ints(rng, shape, lo=-4, hi=5):
    return rng.integers(lo, hi, size=shape).astype(np.float64)


# ------------------------------------------------------------------ MatMul (App. B.1)
def test_matmul_bruteforce_tiny_exact():
    rng = np.random.default_rng(1)
    for (M, N, K) in [(1, 1, 1), (2, 3, 4), (4, 2, 3), (3, 4, 1), (4, 4, 4)]:
        A, B = _ints(rng, (M, K)), _ints(rng, (K, N))
        C = T.matmul(A, B)
        fa, fb = A.ravel().tolist(), B.ravel().tolist()  # flat lists, own index arithmetic
        for i in range(M):
            for j in range(N):
                want = sum(Fraction(fa[i * K + k]) * Fraction(fb[k * N + j]) for k in range(K))
                assert Fraction(C[i, j]) == want, (M, N, K, i, j)


def test_matmul_identity_both_sides():
    rng = np.random.default_rng(2)
    A = rng.standard_normal((5, 7))
    assert np.array_equal(T.matmul(A, np.eye(7)), A)
    assert np.array_equal(T.matmul(np.eye(5), A), A)


def test_matmul_rank1_closed_form():
    # (u v^T)(w z^T) = (v.w) u z^T ; small integers keep every product exact in fp64
    rng = np.random.default_rng(3)
    u, v, w, z = (_ints(rng, n) for n in (6, 9, 9, 5))
    C = T.matmul(np.outer(u, v), np.outer(w, z))
    assert np.array_equal(C, float(v @ w) * np.outer(u, z))


def test_matmul_all_ones_counts_k():
    C = T.matmul(np.ones((3, 37)), np.ones((37, 4)))
    assert np.array_equal(C, np.full((3, 4), 37.0))


def test_matmul_not_transposed():
    # A = e_0 e_1^T (2x3), B = e_1 e_2^T (3x4): only C[0,2] = 1
    A = np.zeros((2, 3)); A[0, 1] = 1
    B = np.zeros((3, 4)); B[1, 2] = 1
    C = T.matmul(A, B)
    want = np.zeros((2, 4)); want[0, 2] = 1
    assert np.array_equal(C, want)


def test_matmul_vs_numpy_float64():
    rng = np.random.default_rng(4)
    A, B = rng.standard_normal((33, 130)), rng.standard_normal((130, 17))
    C = T.matmul(A, B)
    ref = A @ B
    assert np.max(np.abs(C - ref)) <= 1e-12 * np.max(np.abs(ref))


def test_matmul_rows_and_entries_are_the_same_sums():
    rng = np.random.default_rng(5)
    A, B = rng.standard_normal((20, 31)), rng.standard_normal((31, 12))
    C = T.matmul(A, B)
    rows = np.array([19, 0, 7, 7])
    assert np.array_equal(T.matmul_rows(A, B, rows), C[rows])
    is_, js = np.array([0, 19, 3]), np.array([11, 0, 5])
    assert np.array_equal(T.matmul_entries(A, B, is_, js), C[is_, js])


# -------------------------------------------------------------- BatchMatMul (App. B.2)
def test_bmm_bruteforce_tiny_exact():
    rng = np.random.default_rng(6)
    b, M, N, K = 3, 2, 4, 3
    A, B = _ints(rng, (b, M, K)), _ints(rng, (b, K, N))
    C = T.bmm(A, B)
    fa, fb = A.ravel().tolist(), B.ravel().tolist()
    for bb in range(b):
        for i in range(M):
            for j in range(N):
                want = sum(fa[(bb * M + i) * K + k] * fb[(bb * K + k) * N + j] for k in range(K))
                assert C[bb, i, j] == want


def test_bmm_is_per_batch_matmul_and_batches_do_not_mix():
    rng = np.random.default_rng(7)
    A, B = rng.standard_normal((4, 5, 6)), rng.standard_normal((4, 6, 3))
    C = T.bmm(A, B)
    for b in range(4):
        assert np.array_equal(C[b], T.matmul(A[b], B[b]))
    perm = np.array([2, 0, 3, 1])
    assert np.array_equal(T.bmm(A[perm], B[perm]), C[perm])
    # scaling one batch of A by c_b scales only that batch of C (powers of two: exact)
    scale = np.array([1.0, 2.0, 0.5, 4.0])[:, None, None]
    assert np.array_equal(T.bmm(A * scale, B), C * scale)


# --------------------------------------------------------- Conv2d (App. B.3, Eq. 5)
def test_conv_output_extents_golden():
    with open(os.path.join(GOLDEN, "conv_shapes.txt")) as fh:
        rows = [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 4
    for h, k, s, p, want in rows:
        assert T.conv_out_extent(int(h), int(k), int(s), int(p)) == int(want)
    img, ker = np.zeros((1, 1, 9, 12)), np.zeros((2, 1, 3, 5))
    assert T.conv2d(img, ker, stride=2, pad=1).shape == (1, 2, 5, 5)


def test_conv_bruteforce_tiny_exact():
    rng = np.random.default_rng(8)
    for (B, Ci, H, W, Co, Hk, Wk, S, P) in [(1, 1, 3, 3, 1, 3, 3, 1, 1), (2, 3, 5, 4, 2, 3, 2, 1, 0),
                                            (1, 2, 6, 7, 3, 3, 3, 2, 1), (1, 1, 4, 4, 1, 1, 1, 1, 0),
                                            (1, 2, 5, 5, 2, 2, 3, 3, 2)]:
        img, ker = _ints(rng, (B, Ci, H, W)), _ints(rng, (Co, Ci, Hk, Wk))
        out = T.conv2d(img, ker, S, P)
        Ho = (H + 2 * P - Hk) // S + 1
        Wo = (W + 2 * P - Wk) // S + 1
        assert out.shape == (B, Co, Ho, Wo)
        padded = np.zeros((B, Ci, H + 2 * P, W + 2 * P))
        padded[:, :, P:P + H, P:P + W] = img   # explicit zero padding instead of bounds tests
        for b in range(B):
            for co in range(Co):
                for y in range(Ho):
                    for x in range(Wo):
                        want = 0.0
                        for ci in range(Ci):
                            for r in range(Hk):
                                for s in range(Wk):
                                    want += padded[b, ci, y * S + r, x * S + s] * ker[co, ci, r, s]
                        assert out[b, co, y, x] == want


def test_conv_1x1_reduces_to_matmul():
    rng = np.random.default_rng(9)
    img, ker = rng.standard_normal((2, 5, 4, 3)), rng.standard_normal((6, 5, 1, 1))
    out = T.conv2d(img, ker, 1, 0)
    for b in range(2):
        assert np.array_equal(out[b].reshape(6, 12), T.matmul(ker.reshape(6, 5), img[b].reshape(5, 12)))


def test_conv_delta_kernels_identity_and_shift_no_flip():
    rng = np.random.default_rng(10)
    img = rng.standard_normal((1, 1, 5, 6))
    ker = np.zeros((1, 1, 3, 3)); ker[0, 0, 1, 1] = 1
    assert np.array_equal(T.conv2d(img, ker, 1, 1), img)
    # tap (0,0): out[y,x] = in[y-1,x-1] (cross-correlation; a flipped kernel would give in[y+1,x+1])
    ker = np.zeros((1, 1, 3, 3)); ker[0, 0, 0, 0] = 1
    out = T.conv2d(img, ker, 1, 1)
    want = np.zeros_like(img); want[0, 0, 1:, 1:] = img[0, 0, :-1, :-1]
    assert np.array_equal(out, want)
    # tap (2,1): out[y,x] = in[y+1,x]
    ker = np.zeros((1, 1, 3, 3)); ker[0, 0, 2, 1] = 1
    out = T.conv2d(img, ker, 1, 1)
    want = np.zeros_like(img); want[0, 0, :-1, :] = img[0, 0, 1:, :]
    assert np.array_equal(out, want)


def test_conv_all_ones_border_counts():
    Ci = 5
    out = T.conv2d(np.ones((1, Ci, 6, 7)), np.ones((2, Ci, 3, 3)), 1, 1)
    assert np.all(out[:, :, 1:-1, 1:-1] == 9 * Ci)
    assert np.all(out[:, :, 0, 1:-1] == 6 * Ci) and np.all(out[:, :, 1:-1, -1] == 6 * Ci)
    for y, x in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(out[:, :, y, x] == 4 * Ci)


def test_conv_stride_subsamples_stride1_result():
    rng = np.random.default_rng(11)
    img, ker = rng.standard_normal((1, 2, 9, 9)), rng.standard_normal((3, 2, 3, 3))
    full = T.conv2d(img, ker, 1, 1)
    assert np.array_equal(T.conv2d(img, ker, 2, 1), full[:, :, ::2, ::2])
    assert np.array_equal(T.conv2d(img, ker, 4, 1), full[:, :, ::4, ::4])


def test_conv_channels_and_batches_separate():
    # weight only on (co=1, ci=2): output channel 1 sees input channel 2 alone
    rng = np.random.default_rng(12)
    img = rng.standard_normal((2, 3, 4, 4))
    ker = np.zeros((2, 3, 1, 1)); ker[1, 2, 0, 0] = 2.0
    out = T.conv2d(img, ker, 1, 0)
    assert np.all(out[:, 0] == 0) and np.array_equal(out[:, 1], 2.0 * img[:, 2])


@pytest.mark.parametrize("S,P", [(1, 0), (1, 1), (2, 1), (4, 0), (1, 2)])
def test_conv_vs_torch_float64(S, P):
    rng = np.random.default_rng(13)
    img, ker = rng.standard_normal((2, 3, 11, 9)), rng.standard_normal((4, 3, 5, 3))
    ref = torch.nn.functional.conv2d(torch.from_numpy(img), torch.from_numpy(ker), stride=S, padding=P).numpy()
    out = T.conv2d(img, ker, S, P)
    assert out.shape == ref.shape
    assert np.max(np.abs(out - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
