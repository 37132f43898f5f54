"""Pins for the oracle's matrix products, row statistic and scatter (CPU only).

Each test checks the C oracle against something that is not the oracle: a
hand-worked case, pure-Python loops over the printed definition, an explicitly
built projection matrix P, or a closed form.
"""
import itertools

import numpy as np
import pytest

from oracle import ref


def bf16_bits(a):
    """Round-to-nearest-even fp32 -> bf16 bit pattern (uint16), done with integers."""
    u = np.asarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_full_grad_hand_worked_2x2x2():
    # G = dY^T X with dY = [[1,2],[3,4]], X = [[5,6],[7,8]], worked by hand:
    # G[0] = 1*[5,6] + 3*[7,8] = [26,30];  G[1] = 2*[5,6] + 4*[7,8] = [38,44]
    dY = np.array([[1, 2], [3, 4]], np.float32)
    X = np.array([[5, 6], [7, 8]], np.float32)
    G = ref.full_grad(dY, X)
    assert G.tolist() == [[26.0, 30.0], [38.0, 44.0]]
    # a transposed-operand mistake would give X^T dY = [[26,38],[30,44]]
    GC = ref.compressed_grad(dY, X, [1], [0.5])
    assert GC.tolist() == [[19.0, 22.0]]
    # same with dY stored transposed
    assert ref.full_grad(np.ascontiguousarray(dY.T), X, ref.DY_MxT).tolist() == G.tolist()


@pytest.mark.parametrize("dtype", ["f32", "f64", "bf16"])
@pytest.mark.parametrize("layout", [ref.DY_TxM, ref.DY_MxT])
def test_products_vs_python_loops(dtype, layout):
    rng = np.random.default_rng(7)
    T, m, n, r = 9, 7, 5, 6
    dY = rng.standard_normal((T, m)).astype(np.float32)
    X = rng.standard_normal((T, n)).astype(np.float32)
    if dtype == "bf16":
        dYs, Xs = bf16_bits(dY), bf16_bits(X)
        dYv, Xv = bf16_to_f64(dYs), bf16_to_f64(Xs)
    elif dtype == "f64":
        dYs, Xs = dY.astype(np.float64), X.astype(np.float64)
        dYv, Xv = dYs, Xs
    else:
        dYs, Xs = dY, X
        dYv, Xv = dY.astype(np.float64), X.astype(np.float64)
    idx = np.array([0, 2, 2, 3, 6, 6], np.int32)  # duplicates are legal
    rho = rng.uniform(0.5, 2.0, r).astype(np.float32)
    # the printed definition, one scalar at a time
    G_loops = [[sum(dYv[t, k] * Xv[t, i] for t in range(T)) for i in range(n)] for k in range(m)]
    GC_loops = [[float(rho[j]) * sum(dYv[t, idx[j]] * Xv[t, i] for t in range(T))
                 for i in range(n)] for j in range(r)]
    dY_in = dYs if layout == ref.DY_TxM else np.ascontiguousarray(dYs.T)
    G = ref.full_grad(dY_in, Xs, layout)
    GC = ref.compressed_grad(dY_in, Xs, idx, rho, layout)
    np.testing.assert_allclose(G, np.array(G_loops), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(GC, np.array(GC_loops), rtol=1e-13, atol=1e-13)


def test_compressed_grad_is_PT_times_G_with_explicit_P():
    """P^T G with P built as a dense m x r matrix with one nonzero per column (Section 3)."""
    rng = np.random.default_rng(11)
    T, m, n, r = 33, 12, 10, 5
    dY = rng.standard_normal((T, m))
    X = rng.standard_normal((T, n))
    idx = np.array([1, 4, 4, 7, 11], np.int32)
    rho = rng.uniform(0.3, 3.0, r).astype(np.float32)
    P = np.zeros((m, r))
    P[idx, np.arange(r)] = rho
    assert (np.count_nonzero(P, axis=0) == 1).all()
    G_np = dY.T @ X  # library matmul of the printed identity G = dY^T X
    np.testing.assert_allclose(ref.full_grad(dY, X), G_np, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ref.compressed_grad(dY, X, idx, rho), P.T @ G_np, rtol=1e-12,
                               atol=1e-12)


def test_leading_dimensions_are_honoured():
    rng = np.random.default_rng(3)
    T, m, n = 6, 5, 4
    big_dY = rng.standard_normal((T, m + 3)).astype(np.float32)
    big_X = rng.standard_normal((T, n + 2)).astype(np.float32)
    dY, X = big_dY[:, :m], big_X[:, :n]
    G = ref.full_grad(dY, X)
    np.testing.assert_allclose(G, dY.astype(np.float64).T @ X.astype(np.float64), rtol=1e-13)
    big_G = rng.standard_normal((m, n + 5))
    np.testing.assert_allclose(ref.row_stats(big_G[:, :n]), (big_G[:, :n] ** 2).sum(1), rtol=1e-14)


def test_row_stats_closed_form_and_loops():
    m, n = 6, 17
    G = np.array([[float(k + 1)] * n for k in range(m)], np.float32)  # row k is constant k+1
    assert ref.row_stats(G).tolist() == [n * (k + 1) ** 2 for k in range(m)]
    rng = np.random.default_rng(5)
    G = rng.standard_normal((m, n)).astype(np.float32)
    want = [sum(float(G[k, i]) ** 2 for i in range(n)) for k in range(m)]
    np.testing.assert_allclose(ref.row_stats(G), want, rtol=1e-14)
    # sign must not matter, and it is the SQUARED norm (3-4-5 triangle)
    assert ref.row_stats(np.array([[3.0, -4.0]])).tolist() == [25.0]
    bits = bf16_bits(G)
    np.testing.assert_allclose(ref.row_stats(bits), (bf16_to_f64(bits) ** 2).sum(1), rtol=1e-14)


def test_empty_shapes():
    X = np.zeros((0, 4), np.float32)
    dY = np.zeros((0, 3), np.float32)
    assert ref.full_grad(dY, X).tolist() == np.zeros((3, 4)).tolist()
    assert ref.compressed_grad(dY, X, [2], [1.0]).tolist() == [[0.0] * 4]
    assert ref.row_stats(np.zeros((2, 0), np.float32)).tolist() == [0.0, 0.0]
    assert ref.compressed_grad(np.ones((2, 3), np.float32), np.ones((2, 4), np.float32),
                               np.zeros(0, np.int32), np.zeros(0, np.float32)).shape == (0, 4)


def test_bad_index_rejected():
    dY = np.ones((2, 3), np.float32)
    X = np.ones((2, 2), np.float32)
    with pytest.raises(ref.OracleError) as e:
        ref.compressed_grad(dY, X, [3], [1.0])
    assert e.value.code == ref.ERR_SHAPE


def test_scatter_matches_dense_P_update_and_leaves_other_rows():
    """W + alpha P U with P dense (Algorithm 1, last line); duplicates sum."""
    rng = np.random.default_rng(13)
    m, n, r = 9, 6, 5
    W0 = rng.standard_normal((m, n))
    idx = np.array([0, 3, 3, 3, 8], np.int32)
    rho = rng.uniform(0.5, 2.0, r).astype(np.float32)
    U = rng.standard_normal((r, n))
    alpha = 0.25
    P = np.zeros((m, r))
    P[idx, np.arange(r)] = rho
    W = W0.copy()
    ref.scatter_update(W, idx, rho, alpha, U)
    np.testing.assert_allclose(W, W0 + alpha * (P @ U), rtol=1e-14, atol=1e-15)
    untouched = sorted(set(range(m)) - set(idx.tolist()))
    assert (W[untouched] == W0[untouched]).all()  # bit-identical
    # sign and scale: a single row, hand-checkable
    W = np.zeros((2, 2))
    ref.scatter_update(W, [1], [2.0], 0.5, np.array([[1.0, -3.0]]))
    assert W.tolist() == [[0.0, 0.0], [1.0, -3.0]]


def test_reconstruction_identity_for_unit_scale():
    """With rho = 1 and distinct rows, P P^T G keeps the selected rows of G and zeroes the
    rest, so ||P P^T G - G||_F^2 is the sum of the unselected squared row norms (Section 3.2 B)."""
    rng = np.random.default_rng(17)
    T, m, n = 20, 8, 6
    dY = rng.standard_normal((T, m))
    X = rng.standard_normal((T, n))
    G = ref.full_grad(dY, X)
    ss = ref.row_stats(G)
    for sel in itertools.combinations(range(m), 3):
        idx = np.array(sel, np.int32)
        GC = ref.compressed_grad(dY, X, idx, np.ones(3, np.float32))
        recon = np.zeros_like(G)
        ref.scatter_update(recon, idx, np.ones(3, np.float32), 1.0, GC)  # P (P^T G)
        err = ((recon - G) ** 2).sum()
        rest = sorted(set(range(m)) - set(sel))
        np.testing.assert_allclose(err, ss[rest].sum(), rtol=1e-12)


def test_column_projection_is_the_transposed_problem():
    """Projecting the columns of G (Section 4.1 projects the smaller dimension) with an n x r matrix P:
    G P = (P^T G^T)^T, and G^T = X^T dY is the gradient of the transposed layer, so the
    compressed gradient is the row form with dY and X exchanged; the update is W + alpha (P U)^T."""
    rng = np.random.default_rng(41)
    T, m, n, r = 25, 9, 6, 4
    dY = rng.standard_normal((T, m))
    X = rng.standard_normal((T, n))
    W0 = rng.standard_normal((m, n))
    idx = np.array([0, 2, 2, 5], np.int32)  # columns of W, one duplicate
    rho = rng.uniform(0.5, 2.0, r).astype(np.float32)
    P = np.zeros((n, r))
    P[idx, np.arange(r)] = rho
    G = dY.T @ X
    GC = ref.compressed_grad(X, dY, idx, rho)  # r x m
    np.testing.assert_allclose(GC, (G @ P).T, rtol=1e-12, atol=1e-13)
    U = rng.standard_normal((r, m))
    W = W0.copy()
    ref.scatter_update_cols(W, idx, rho, 0.25, U)
    np.testing.assert_allclose(W, W0 + 0.25 * (P @ U).T, rtol=1e-14, atol=1e-15)
    untouched = sorted(set(range(n)) - set(idx.tolist()))
    assert (W[:, untouched] == W0[:, untouched]).all()
    # hand-checkable: one column, two rows
    W = np.zeros((2, 3))
    ref.scatter_update_cols(W, [2], [2.0], 0.5, np.array([[1.0, -3.0]]))
    assert W.tolist() == [[0.0, 0.0, 1.0], [0.0, 0.0, -3.0]]
    with pytest.raises(ref.OracleError):
        ref.scatter_update_cols(np.zeros((2, 3)), [3], [1.0], 1.0, np.zeros((1, 2)))
