"""Pins for the oracle's compute_P (Section 3.2) and its random-number generator (CPU only)."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def paper_value(key):
    for line in open(os.path.join(GOLDEN, "paper_values.txt")):
        if line.startswith(key + " "):
            return float(line.split()[1])
    raise KeyError(key)


# ----------------------------------------------------------------------------- RNG
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        out = ref.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def philox4x32_10_from_the_round_definition(ctr, key):
    """Philox4x32-10 restated from the round function of Salmon et al. (SC'11, Section 3.3 and
    Table 2) with Python integers: one round multiplies counter words 0 and 2 by the two
    multipliers (full 64-bit products), crosses the halves over, and xors the high halves with
    the other two words and the round key; the key is bumped by the Weyl constants between
    rounds.  The Weyl constants are not typed in: they are the golden ratio and sqrt(3) - 1 as
    32-bit fractions, computed here with integer square roots."""
    from math import isqrt
    w0 = (isqrt(5 << 64) - (1 << 32)) // 2          # floor(2^32 (sqrt(5) - 1) / 2)
    w1 = isqrt(3 << 64) - (1 << 32)                 # floor(2^32 (sqrt(3) - 1))
    assert (w0, w1) == (0x9E3779B9, 0xBB67AE85)
    m0, m1 = 0xD2511F53, 0xCD9E8D57                  # the paper's multipliers for 4 x 32
    c, k = [int(x) for x in ctr], [int(x) for x in key]
    for rnd in range(10):
        if rnd:
            k = [(k[0] + w0) & 0xFFFFFFFF, (k[1] + w1) & 0xFFFFFFFF]
        p0, p1 = m0 * c[0], m1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
    return c


def test_philox_equals_a_big_integer_restatement_of_the_round_definition():
    rows = [[int(x, 16) for x in l.split()] for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    for v in rows:  # the restatement reproduces the published vectors by itself
        assert philox4x32_10_from_the_round_definition(v[0:4], v[4:6]) == v[6:10]
    rng = np.random.default_rng(1976)
    for _ in range(300):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2)]
        assert [int(x) for x in ref.philox4x32_10(ctr, key)] == philox4x32_10_from_the_round_definition(ctr, key)


def test_third_known_answer_vector_is_keyed_by_the_digits_of_pi():
    """The published vectors use the fractional hexadecimal digits of pi as the third counter
    and key; that part of the fixture can be derived instead of recalled.  pi from Machin's
    formula in integer arithmetic."""
    bits = 192 + 64

    def arctan_inv(x):  # 2^bits * arctan(1 / x)
        total, term, n, sign = 0, (1 << bits) // x, 1, 1
        while term:
            total += sign * (term // n)
            term //= x * x
            n += 2
            sign = -sign
        return total
    pi = 4 * (4 * arctan_inv(5) - arctan_inv(239))
    frac = (pi - (3 << bits)) >> 64  # the first 192 fractional bits
    words = [(frac >> (160 - 32 * i)) & 0xFFFFFFFF for i in range(6)]
    rows = [[int(x, 16) for x in l.split()] for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert rows[2][:6] == words


def test_draw_word_packing():
    seed, refresh, j = 0x0123456789ABCDEF, 0xFEDCBA9876543210, 0x1122334455667788
    out = ref.philox4x32_10([j & 0xFFFFFFFF, j >> 32, refresh & 0xFFFFFFFF, refresh >> 32],
                            [seed & 0xFFFFFFFF, seed >> 32])
    assert ref.draw_word(seed, refresh, j) == int(out[0]) | (int(out[1]) << 32)
    # distinct draws, refreshes and seeds give distinct words
    words = {ref.draw_word(s, f, k) for s in range(3) for f in range(3) for k in range(50)}
    assert len(words) == 3 * 3 * 50


def test_draw_words_look_uniform():
    x = np.array([ref.draw_word(42, 7, j) for j in range(20000)], dtype=np.uint64)
    u = x.astype(np.float64) / 2.0 ** 64
    assert abs(u.mean() - 0.5) < 4 / np.sqrt(12 * len(u))
    counts = np.bincount((x >> np.uint64(60)).astype(np.int64), minlength=16)
    chi2 = ((counts - len(u) / 16) ** 2 / (len(u) / 16)).sum()
    assert chi2 < 45  # 15 dof, p ~ 1e-4
    for bit in (0, 17, 31, 32, 47, 63):
        ones = int(((x >> np.uint64(bit)) & np.uint64(1)).sum())
        assert abs(ones - len(u) / 2) < 4 * np.sqrt(len(u)) / 2


def test_mulhi64_vs_bigint():
    rng = np.random.default_rng(1)
    cases = [(0, 0), (2 ** 64 - 1, 2 ** 64 - 1), (2 ** 63, 2), (1, 2 ** 64 - 1)]
    cases += [(int(a), int(b)) for a, b in rng.integers(0, 2 ** 64, (200, 2), dtype=np.uint64)]
    for a, b in cases:
        assert ref.mulhi64(a, b) == (a * b) >> 64


# ----------------------------------------------------------------------------- weights
def test_sampling_weights_properties():
    rng = np.random.default_rng(2)
    ss = (rng.standard_normal(50) ** 2 * 10).astype(np.float32)
    one = 2 ** 40
    wu = ref.sampling_weights(ss, ref.UNIFORM)
    assert (wu == one + 1).all()
    w1 = ref.sampling_weights(ss, ref.MULTI_NORM).astype(np.float64)
    w2 = ref.sampling_weights(ss, ref.MULTI_NORM2).astype(np.float64)
    k = int(np.argmax(ss))
    assert w1[k] == one + 1 and w2[k] == one + 1
    s = ss.astype(np.float64)
    # q_k proportional to the norm (Theorem 3.1) resp. the squared norm, on a 2^-40 grid
    np.testing.assert_allclose((w1 - 1) / one, np.sqrt(s / s[k]), atol=2.0 ** -39)
    np.testing.assert_allclose((w2 - 1) / one, s / s[k], atol=2.0 ** -39)
    assert (w1 >= 1).all() and (w2 >= 1).all()
    order = np.argsort(ss, kind="stable")
    assert (np.diff(w1[order]) >= 0).all() and (np.diff(w2[order]) >= 0).all()
    # all-zero gradient: every row equally likely
    assert (ref.sampling_weights(np.zeros(5, np.float32), ref.MULTI_NORM) == 1).all()
    # a zero row keeps a nonzero probability
    z = ref.sampling_weights(np.array([0.0, 4.0], np.float32), ref.MULTI_NORM)
    assert z.tolist() == [1, one + 1]
    # exactly representable ratios: norms 1 : 2 : 4
    e = ref.sampling_weights(np.array([1.0, 4.0, 16.0], np.float32), ref.MULTI_NORM)
    assert e.tolist() == [one // 4 + 1, one // 2 + 1, one + 1]
    e2 = ref.sampling_weights(np.array([1.0, 4.0, 16.0], np.float32), ref.MULTI_NORM2)
    assert e2.tolist() == [one // 16 + 1, one // 4 + 1, one + 1]


@pytest.mark.parametrize("bad", [np.nan, np.inf, -1.0])
def test_nonfinite_rejected(bad):
    ss = np.array([1.0, bad, 2.0], np.float32)
    for method in (ref.TOPR, ref.UNIFORM, ref.MULTI_NORM):
        with pytest.raises(ref.OracleError) as e:
            ref.select_rows(ss, 1, method)
        assert e.value.code == ref.ERR_NONFINITE


# ----------------------------------------------------------------------------- Top-r
def test_topr_equals_argsort_without_ties():
    rng = np.random.default_rng(3)
    for m, r in [(1, 1), (7, 3), (64, 64), (200, 17), (1000, 999)]:
        ss = rng.permutation(m).astype(np.float32) + 0.5  # all distinct
        idx, rho, _ = ref.select_rows(ss, r, ref.TOPR)
        want = np.sort(np.argsort(-ss.astype(np.float64), kind="stable")[:r])
        assert idx.tolist() == want.tolist()
        assert (rho == 1.0).all()
        assert (np.diff(idx) > 0).all()


def test_topr_ties_go_to_lower_index_and_negative_zero_is_zero():
    ss = np.array([2.0, 5.0, 2.0, 5.0, 2.0, 1.0], np.float32)
    assert ref.select_rows(ss, 1, ref.TOPR)[0].tolist() == [1]
    assert ref.select_rows(ss, 3, ref.TOPR)[0].tolist() == [0, 1, 3]
    assert ref.select_rows(ss, 4, ref.TOPR)[0].tolist() == [0, 1, 2, 3]
    ss = np.array([-0.0, 0.0, 1e-45, 0.0], np.float32)  # -0 must not outrank a denormal
    assert ref.select_rows(ss, 2, ref.TOPR)[0].tolist() == [0, 2]


def test_topr_minimises_reconstruction_error_over_all_subsets():
    """Section 3.2 B: Top-r minimises ||P P^T G - G||_F^2 among selections with rho = 1."""
    rng = np.random.default_rng(4)
    for m, r in [(6, 2), (9, 4), (12, 5)]:
        G = rng.standard_normal((m, 5)) * rng.uniform(0.1, 3.0, (m, 1))
        ss = (G ** 2).sum(1).astype(np.float32)
        idx, _, _ = ref.select_rows(ss, r, ref.TOPR)

        def err(sel):
            P = np.zeros((m, r))
            P[list(sel), np.arange(r)] = 1.0
            return ((P @ P.T @ G - G) ** 2).sum()

        best = min(itertools.combinations(range(m), r), key=err)
        assert tuple(idx.tolist()) == best


def test_structure_of_P():
    """Each column of P has exactly one nonzero; 0 <= idx < m; idx ascending."""
    rng = np.random.default_rng(5)
    ss = (rng.standard_normal(40) ** 2).astype(np.float32)
    for method, repl in [(ref.TOPR, False), (ref.UNIFORM, True), (ref.UNIFORM, False),
                         (ref.MULTI_NORM, True), (ref.MULTI_NORM, False),
                         (ref.MULTI_NORM2, True), (ref.MULTI_NORM2, False)]:
        idx, rho, _ = ref.select_rows(ss, 25, method, repl, seed=9, refresh_id=1)
        assert idx.min() >= 0 and idx.max() < 40
        assert (np.diff(idx) >= 0).all()
        assert (rho > 0).all() and np.isfinite(rho).all()
        if method == ref.TOPR or not repl:
            assert (np.diff(idx) > 0).all()  # a row is used by at most one column
            assert (rho == 1.0).all()  # Section 3.2: rho = 1 for NR and Top-r


def test_shape_errors():
    ss = np.ones(4, np.float32)
    for method, repl in [(ref.TOPR, False), (ref.UNIFORM, False)]:
        with pytest.raises(ref.OracleError) as e:
            ref.select_rows(ss, 5, method, repl)
        assert e.value.code == ref.ERR_SHAPE
    assert len(ref.select_rows(ss, 9, ref.UNIFORM, True)[0]) == 9  # iid draws may exceed m
    with pytest.raises(ref.OracleError) as e:
        ref.select_rows(ss, 2, ref.TOPR, False, ref.SCALE_INV_SQRT_RQ)
    assert e.value.code == ref.ERR_DTYPE
    assert len(ref.select_rows(ss, 0, ref.TOPR)[0]) == 0


# ----------------------------------------------------------------------------- sampling
def python_sampler(wq, r, replacement, seed, refresh):
    """The draw rule with Python integers: an independent brute-force restatement."""
    w = [int(x) for x in wq]
    out = []
    for j in range(r):
        remaining = sum(w)
        target = (ref.draw_word(seed, refresh, j) * remaining) >> 64
        c = 0
        for k, wk in enumerate(w):
            c += wk
            if c > target:
                out.append(k)
                break
        if not replacement:
            w[out[-1]] = 0
    return sorted(out)


@pytest.mark.parametrize("method", [ref.UNIFORM, ref.MULTI_NORM, ref.MULTI_NORM2])
@pytest.mark.parametrize("replacement", [True, False])
def test_sampler_vs_bigint_restatement(method, replacement):
    rng = np.random.default_rng(6)
    for m, r in [(1, 1), (5, 5), (37, 11), (300, 120)]:
        ss = (rng.standard_normal(m) ** 2).astype(np.float32)
        ss[rng.integers(0, m)] = 0.0
        wq = ref.sampling_weights(ss, method)
        for seed, refresh in [(0, 0), (123456789012345, 3)]:
            idx, _, _ = ref.select_rows(ss, r, method, replacement, seed=seed, refresh_id=refresh)
            assert idx.tolist() == python_sampler(wq, r, replacement, seed, refresh)


def test_with_replacement_frequencies_follow_q():
    ss = np.array([1.0, 4.0, 9.0, 16.0, 0.25], np.float32)  # norms 1,2,3,4,0.5
    q = np.array([1, 2, 3, 4, 0.5]) / 10.5
    r, N = 8, 4000
    counts = np.zeros(5)
    for s in range(N):
        idx, _, _ = ref.select_rows(ss, r, ref.MULTI_NORM, True, seed=s, refresh_id=0)
        counts += np.bincount(idx, minlength=5)
    expect = q * r * N
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 24  # 4 dof, p ~ 1e-4
    # squared-norm rule
    q2 = np.array([1, 4, 9, 16, 0.25]) / 30.25
    counts = np.zeros(5)
    for s in range(N):
        counts += np.bincount(ref.select_rows(ss, r, ref.MULTI_NORM2, True, seed=s)[0], minlength=5)
    assert (((counts - q2 * r * N) ** 2) / (q2 * r * N)).sum() < 24


def test_rho_satisfies_r_q_rho2_equals_1():
    """Section 3.2 A: rho_jj = 1 / sqrt(r q_sigma_j)."""
    rng = np.random.default_rng(8)
    ss = (rng.standard_normal(30) ** 2).astype(np.float32)
    for method in (ref.UNIFORM, ref.MULTI_NORM, ref.MULTI_NORM2):
        wq = [int(x) for x in ref.sampling_weights(ss, method)]
        total = sum(wq)
        idx, rho, rho_d = ref.select_rows(ss, 12, method, True, seed=5)
        for j in range(12):
            q = Fraction(wq[idx[j]], total)
            assert abs(12 * float(q) * rho_d[j] ** 2 - 1.0) < 1e-14
            assert rho[j] == np.float32(rho_d[j])
        # NR with the forced rescale uses the q of the initial distribution
        idx, rho, rho_d = ref.select_rows(ss, 12, method, False, ref.SCALE_INV_SQRT_RQ, seed=5)
        for j in range(12):
            assert abs(12 * wq[idx[j]] / total * rho_d[j] ** 2 - 1.0) < 1e-14
        # and the forced unit scale
        assert (ref.select_rows(ss, 12, method, True, ref.SCALE_ONE, seed=5)[1] == 1.0).all()
    # uniform: rho = sqrt(m / r)
    _, _, rho_d = ref.select_rows(ss, 12, ref.UNIFORM, True)
    np.testing.assert_allclose(rho_d, np.sqrt(30 / 12), rtol=1e-15)


@pytest.mark.parametrize("method", [ref.UNIFORM, ref.MULTI_NORM, ref.MULTI_NORM2])
def test_unbiasedness_and_total_variance(method):
    """Appendix D: E[P P^T G] = G.  Appendix E: total variance =
    (1/r) (sum_k ||G_k||^2 / q_k - ||G||_F^2)."""
    rng = np.random.default_rng(10)
    m, n, r, N = 12, 3, 4, 30000
    G = rng.standard_normal((m, n)) * rng.uniform(0.2, 2.0, (m, 1))
    ss64 = (G ** 2).sum(1)
    ss = ss64.astype(np.float32)
    wq = ref.sampling_weights(ss, method).astype(np.float64)
    q = wq / wq.sum()
    var_closed = ((ss64 / q).sum() - ss64.sum()) / r
    mean = np.zeros_like(G)
    sq_err = 0.0
    for s in range(N):
        idx, _, rho_d = ref.select_rows(ss, r, method, True, seed=1000 + s, refresh_id=2)
        P = np.zeros((m, r))
        P[idx, np.arange(r)] = rho_d
        est = P @ (P.T @ G)
        mean += est
        sq_err += ((est - G) ** 2).sum()
    mean /= N
    fro = np.sqrt(ss64.sum())
    assert np.linalg.norm(mean - G) / fro < 4 * np.sqrt(var_closed / N) / fro
    assert abs(sq_err / N / var_closed - 1.0) < 0.06


def test_norm_sampling_has_least_variance():
    """Theorem 3.1, through the closed form of Appendix E evaluated on the oracle's q."""
    rng = np.random.default_rng(12)
    ss64 = (rng.standard_normal(50) * rng.uniform(0.1, 4, 50)) ** 2
    ss = ss64.astype(np.float32)
    ss64 = ss.astype(np.float64)

    def var(method):
        wq = ref.sampling_weights(ss, method).astype(np.float64)
        q = wq / wq.sum()
        return (ss64 / q).sum() - ss64.sum()

    lam = np.sqrt(ss64)
    np.testing.assert_allclose(var(ref.MULTI_NORM), lam.sum() ** 2 - (lam ** 2).sum(), rtol=1e-9)
    np.testing.assert_allclose(var(ref.UNIFORM), (50 - 1) * ss64.sum(), rtol=1e-9)
    assert var(ref.MULTI_NORM) < var(ref.UNIFORM)
    assert var(ref.MULTI_NORM) < var(ref.MULTI_NORM2)


def test_uniform_coverage_matches_printed_value():
    """The paper's coverage paragraph: m = 512, r = 128, 15 refreshes, uniform with
    replacement -> 97.66 % of rows touched on average."""
    printed = paper_value("uniform_coverage_m512_r128_n15_percent")
    assert abs(100 * (1 - ((1 - 1 / 512) ** 128) ** 15) - printed) < 0.005
    ss = np.ones(512, np.float32)
    cov = []
    for trial in range(200):
        seen = set()
        for refresh in range(15):
            idx, _, _ = ref.select_rows(ss, 128, ref.UNIFORM, True, seed=trial, refresh_id=refresh)
            seen.update(idx.tolist())
        cov.append(len(seen) / 512 * 100)
    # std of one trial's coverage ~ 0.66 %, of the mean of 200 ~ 0.05 %
    assert abs(np.mean(cov) - printed) < 0.2


# ----------------------------------------------------------------------------- without replacement
def test_nr_special_cases():
    rng = np.random.default_rng(14)
    ss = (rng.standard_normal(20) ** 2).astype(np.float32)
    for method in (ref.UNIFORM, ref.MULTI_NORM, ref.MULTI_NORM2):
        for seed in range(20):
            # one draw: with and without replacement coincide
            assert (ref.select_rows(ss, 1, method, False, seed=seed)[0].tolist()
                    == ref.select_rows(ss, 1, method, True, seed=seed)[0].tolist())
            # r = m: every row exactly once
            assert ref.select_rows(ss, 20, method, False, seed=seed)[0].tolist() == list(range(20))
            idx = ref.select_rows(ss, 13, method, False, seed=seed)[0]
            assert len(set(idx.tolist())) == 13


def test_nr_inclusion_probabilities_vs_exact_enumeration():
    """m = 4, r = 2: inclusion probability of each row under sequential draw-and-remove,
    enumerated exactly from q, against the oracle's empirical frequencies."""
    ss = np.array([1.0, 4.0, 9.0, 36.0], np.float32)  # norms 1, 2, 3, 6
    wq = [int(x) for x in ref.sampling_weights(ss, ref.MULTI_NORM)]
    total = sum(wq)
    incl = [Fraction(0)] * 4
    for a in range(4):
        for b in range(4):
            if a == b:
                continue
            p = Fraction(wq[a], total) * Fraction(wq[b], total - wq[a])
            incl[a] += p
            incl[b] += p
    assert sum(incl) == 2
    N = 20000
    counts = np.zeros(4)
    for s in range(N):
        counts += np.bincount(ref.select_rows(ss, 2, ref.MULTI_NORM, False, seed=s)[0], minlength=4)
    for k in range(4):
        p = float(incl[k])
        assert abs(counts[k] / N - p) < 4.5 * np.sqrt(p * (1 - p) / N)
