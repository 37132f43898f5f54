"""Pins for the oracle's Adam update and for the whole step (CPU only)."""
import numpy as np
import torch

from oracle import ref

LR, B1, B2, EPS = 1e-3, 0.9, 0.999, 1e-8  # Adam defaults the paper states (Appendix I)


def test_adam_first_step_closed_form():
    """At t = 1 with zero state the bias corrections cancel:
    M = (1-b1) g, V = (1-b2) g^2, U = -lr * g / (|g| + eps)."""
    g = np.array([[0.5, -2.0, 0.0, 1e-6], [3.0, -1e-3, 7.0, -0.25]])
    M = np.zeros_like(g)
    V = np.zeros_like(g)
    U = ref.adam_rows(g, M, V, LR, B1, B2, EPS, 1)
    np.testing.assert_allclose(M, (1 - B1) * g, rtol=1e-15)
    np.testing.assert_allclose(V, (1 - B2) * g * g, rtol=1e-15)
    np.testing.assert_allclose(U, -LR * g / (np.abs(g) + EPS), rtol=1e-12, atol=0)
    assert U[0, 2] == 0.0
    assert (np.sign(U) == -np.sign(g)).all()  # the update opposes the gradient


def test_adam_second_step_by_hand():
    """Two steps on one scalar, every intermediate written out with the numbers themselves
    (lr = 0.1, b1 = 0.5, b2 = 0.75, eps = 0, g1 = 2, g2 = 4)."""
    M = np.zeros((1, 1))
    V = np.zeros((1, 1))
    U1 = ref.adam_rows(np.array([[2.0]]), M, V, 0.1, 0.5, 0.75, 0.0, 1)
    assert M[0, 0] == 1.0 and V[0, 0] == 1.0  # 0.5*2, 0.25*4
    np.testing.assert_allclose(U1, [[-0.1]], rtol=1e-15)  # -0.1 * (1/0.5) / sqrt(1/0.25)
    U2 = ref.adam_rows(np.array([[4.0]]), M, V, 0.1, 0.5, 0.75, 0.0, 2)
    assert M[0, 0] == 2.5  # 0.5*1 + 0.5*4
    assert V[0, 0] == 4.75  # 0.75*1 + 0.25*16
    # M* = 2.5/(1-0.25) = 10/3 ; V* = 4.75/(1-0.5625) = 76/7 ; U = -0.1*(10/3)/sqrt(76/7)
    np.testing.assert_allclose(U2, [[-0.1 * (10 / 3) / np.sqrt(76 / 7)]], rtol=1e-15)


def test_adam_matches_library_adam_over_several_steps():
    """torch.optim.Adam (no weight decay, no amsgrad) applies p += U with the same U."""
    rng = np.random.default_rng(21)
    r, n = 5, 7
    p = torch.zeros(r, n, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=LR, betas=(B1, B2), eps=EPS)
    M = np.zeros((r, n))
    V = np.zeros((r, n))
    acc = np.zeros((r, n))
    for t in range(1, 8):
        g = rng.standard_normal((r, n)) * 10.0 ** rng.integers(-3, 3)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        acc += ref.adam_rows(g, M, V, LR, B1, B2, EPS, t)
        np.testing.assert_allclose(acc, p.detach().numpy(), rtol=1e-10, atol=1e-16)
    st = opt.state[p]
    np.testing.assert_allclose(M, st["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(V, st["exp_avg_sq"].numpy(), rtol=1e-12)


def test_adam_leading_dimension_and_errors():
    rng = np.random.default_rng(22)
    big = rng.standard_normal((3, 9))
    M1, V1 = np.zeros((3, 4)), np.zeros((3, 4))
    M2, V2 = np.zeros((3, 4)), np.zeros((3, 4))
    U1 = ref.adam_rows(big[:, :4], M1, V1, LR, B1, B2, EPS, 1)
    U2 = ref.adam_rows(np.ascontiguousarray(big[:, :4]), M2, V2, LR, B1, B2, EPS, 1)
    assert (U1 == U2).all() and (M1 == M2).all() and (V1 == V2).all()
    for bad_t in (0, -1):
        try:
            ref.adam_rows(big[:, :4], M1, V1, LR, B1, B2, EPS, bad_t)
            assert False
        except ref.OracleError as e:
            assert e.code == ref.ERR_SHAPE


def test_all_rows_selected_is_dense_adam():
    """r = m, sigma = identity, rho = 1, alpha = 1: the GRASS step is the full-rank update of
    Eq. (1), W <- W + opt.update(grad).  The dense side is torch's Adam fed numpy's dY^T X."""
    rng = np.random.default_rng(23)
    T, m, n = 40, 6, 5
    W0 = rng.standard_normal((m, n))
    p = torch.tensor(W0.copy(), requires_grad=True)
    opt = torch.optim.Adam([p], lr=LR, betas=(B1, B2), eps=EPS)
    W = W0.copy()
    M = np.zeros((m, n))
    V = np.zeros((m, n))
    idx = np.arange(m, dtype=np.int32)
    rho = np.ones(m, np.float32)
    for t in range(1, 4):
        dY = rng.standard_normal((T, m))
        X = rng.standard_normal((T, n))
        p.grad = torch.from_numpy(dY.T @ X)
        opt.step()
        GC = ref.compressed_grad(dY, X, idx, rho)
        U = ref.adam_rows(GC, M, V, LR, B1, B2, EPS, t)
        ref.scatter_update(W, idx, rho, 1.0, U)
        np.testing.assert_allclose(W, p.detach().numpy(), rtol=1e-11, atol=1e-14)


def test_sparse_step_equals_dense_formulation_with_explicit_P():
    """One step of Algorithm 1 written with dense matrices: G_C = P^T G, Delta = Adam(G_C),
    W + alpha P Delta, for a sampled P with duplicates and non-unit rho."""
    rng = np.random.default_rng(24)
    T, m, n, r = 30, 10, 4, 6
    dY = rng.standard_normal((T, m))
    X = rng.standard_normal((T, n))
    W0 = rng.standard_normal((m, n))
    G = dY.T @ X
    ss = (G ** 2).sum(1).astype(np.float32)
    idx, rho, _ = ref.select_rows(ss, r, ref.MULTI_NORM, True, seed=3)
    P = np.zeros((m, r))
    P[idx, np.arange(r)] = rho.astype(np.float64)
    GC_dense = P.T @ G
    p = torch.zeros(r, n, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=LR, betas=(B1, B2), eps=EPS)
    p.grad = torch.from_numpy(GC_dense)
    opt.step()
    W_dense = W0 + 0.25 * P @ p.detach().numpy()

    GC = ref.compressed_grad(dY, X, idx, rho)
    M, V = np.zeros((r, n)), np.zeros((r, n))
    U = ref.adam_rows(GC, M, V, LR, B1, B2, EPS, 1)
    W = W0.copy()
    ref.scatter_update(W, idx, rho, 0.25, U)
    np.testing.assert_allclose(GC, GC_dense, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(W, W_dense, rtol=1e-11, atol=1e-14)


# ------------------------------------------------------------------------------ bf16 moments
def exact_bf16(x):
    """Round a float to 8 significant bits, ties to even, in exact rational arithmetic."""
    from fractions import Fraction
    if x == 0.0:
        return 0.0
    fx = Fraction(x)
    e = 0
    while abs(fx) >= Fraction(2) ** e:
        e += 1
    while abs(fx) < Fraction(2) ** (e - 1):
        e -= 1
    q = Fraction(2) ** max(e - 8, -133)
    k = fx / q
    lo = k.numerator // k.denominator  # floor
    rem = k - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return float(lo * q)


def test_round_bf16_against_exact_rational_rounding_and_bit_patterns():
    rng = np.random.default_rng(31)
    xs = np.concatenate([rng.standard_normal(200) * 10.0 ** rng.integers(-20, 20, 200),
                         [1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40,
                          -(1.0 + 2.0 ** -8), 255.5, 256.5, 2.0 ** -126, 3 * 2.0 ** -134, 0.0]])
    got = ref.round_bf16(xs)
    assert got.tolist() == [exact_bf16(float(x)) for x in xs]
    # ties go to the even neighbour: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert got[201] == 1.0 and got[202] == 1.0 + 2.0 ** -6 and got[203] == 1.0 + 2.0 ** -7
    # the results are bf16 values: fp32 bit patterns with 16 zero low bits
    bits = got.astype(np.float32).view(np.uint32)
    assert (got.astype(np.float32) == got).all() and ((bits & 0xFFFF) == 0).all()
    # fp32 inputs: same as the integer rounding of the bit pattern
    f = rng.standard_normal(500).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    want = (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16).astype(np.uint32).view(np.float32)
    assert (ref.round_bf16(f) == want).all()


def test_adam_bf16_state_python_loop_with_exact_rounding():
    """Moments rounded once per step, the update computed from the rounded moments."""
    rng = np.random.default_rng(32)
    r, n = 3, 4
    M = np.zeros((r, n))
    V = np.zeros((r, n))
    Mp = [[0.0] * n for _ in range(r)]
    Vp = [[0.0] * n for _ in range(r)]
    for t in range(1, 5):
        g = rng.standard_normal((r, n)) * 0.3
        U = ref.adam_rows(g, M, V, LR, B1, B2, EPS, t, state_bf16=True)
        for j in range(r):
            for i in range(n):
                Mp[j][i] = exact_bf16(B1 * Mp[j][i] + (1 - B1) * g[j, i])
                Vp[j][i] = exact_bf16(B2 * Vp[j][i] + (1 - B2) * g[j, i] * g[j, i])
                u = -LR * (Mp[j][i] / (1 - B1 ** t)) / ((Vp[j][i] / (1 - B2 ** t)) ** 0.5 + EPS)
                assert M[j, i] == Mp[j][i] and V[j, i] == Vp[j][i]
                np.testing.assert_allclose(U[j, i], u, rtol=1e-13)
    # the rounding is really there: the fp64 moments of the same sequence differ
    M64 = np.zeros((r, n))
    V64 = np.zeros((r, n))
    rng = np.random.default_rng(32)
    for t in range(1, 5):
        ref.adam_rows(rng.standard_normal((r, n)) * 0.3, M64, V64, LR, B1, B2, EPS, t)
    assert np.abs(M - M64).max() > 0 and np.abs(M - M64).max() <= 2.0 ** -7 * np.abs(M64).max()


def test_adam_bf16_state_equals_fp64_adam_when_nothing_needs_rounding():
    """b1 = b2 = 0.5 and power-of-two gradients keep every moment exactly representable."""
    g1 = np.array([[2.0, -4.0, 0.5]])
    g2 = np.array([[1.0, 8.0, -0.25]])
    Ma, Va, Mb, Vb = (np.zeros((1, 3)) for _ in range(4))
    for t, g in ((1, g1), (2, g2)):
        Ua = ref.adam_rows(g, Ma, Va, 0.1, 0.5, 0.5, 0.0, t)
        Ub = ref.adam_rows(g, Mb, Vb, 0.1, 0.5, 0.5, 0.0, t, state_bf16=True)
        assert (Ua == Ub).all() and (Ma == Mb).all() and (Va == Vb).all()
    assert Mb.tolist() == [[1.0, 3.0, 0.0]]  # 0.5*(0.5*g1) + 0.5*g2
