"""Pins for the CPU oracle: everything here checks oracle/ against something other than itself --
the paper's worked example, numpy's Kronecker product and matmul, closed forms and algebraic
identities.  No GPU is needed.

The checks are written as functions of an implementation `impl(X, Fs) -> Y` so that the same suite
can be turned on deliberately broken variants (test_pins_catch_planted_mistakes): each plausible
slip -- transposed factor, reversed factor order, wrong output digit order, dropped term -- must be
rejected by at least one pin.
"""
import numpy as np
import pytest

import oracle
import kron_inputs
from conftest import read_golden


def kron_all(Fs):
    G = np.asarray(Fs[0], dtype=np.float64)
    for F in Fs[1:]:
        G = np.kron(G, np.asarray(F, dtype=np.float64))
    return G


def small_int_problem(M, shapes, seed, dtype=np.float64):
    return kron_inputs.make_problem(M, shapes, dtype, "int2", "int2", seed)


# ---------------------------------------------------------------- pins as reusable checks

def check_worked_example(impl):
    """Figure 2 (first iteration of the 2x4 example), through a one-factor call per slice layout:
    with F1 = identity the whole product equals the first-iteration matrix re-read by iteration 2,
    so use the dedicated single-iteration entry when impl is the oracle; here: full product with
    both factors against the printed first-iteration values pushed through F1 by hand."""
    g = read_golden("fig2_first_iteration_2x4.txt")
    X = np.array(g["x"]).reshape(2, 4)
    F2 = np.array(g["f2"]).reshape(2, 2)
    Y2 = np.array(g["y2"]).reshape(2, 4)
    # second iteration by the same printed rule, with F1 = [[1, -1], [2, 1]] worked by hand:
    # Y1[r] = [y_r1 a11 + y_r2 a21, y_r3 a11 + y_r4 a21, y_r1 a12 + y_r2 a22, y_r3 a12 + y_r4 a22]
    F1 = np.array([[1.0, -1.0], [2.0, 1.0]])
    Y1 = np.array([[7 + 30, 10 + 44, -7 + 15, -10 + 22],
                   [23 + 62, 34 + 92, -23 + 31, -34 + 46]], dtype=np.float64)
    assert np.array_equal(impl(X, [F1, F2]), Y1)
    # and F1 = I leaves iteration 2 as the inverse shuffle of iteration 1: columns (q, s) -> (s, q)
    Yi = impl(X, [np.eye(2), F2])
    assert np.array_equal(Yi, Y2.reshape(2, 2, 2).transpose(0, 2, 1).reshape(2, 4))


def check_against_numpy_kron(impl, dtype=np.float64):
    cases = [
        (3, [(2, 2), (2, 2)]),
        (1, [(3, 2)]),                       # N = 1: plain X @ F
        (4, [(2, 3), (4, 2), (3, 5)]),       # distinct rectangular factors
        (2, [(1, 3), (4, 1), (2, 2)]),       # P = 1 and Q = 1 factors
        (5, [(8, 8), (8, 8), (8, 8)]),
        (2, [(5, 3), (2, 7)]),
        (1, [(1, 1), (1, 1)]),
    ]
    for seed, (M, shapes) in enumerate(cases):
        X, Fs = small_int_problem(M, shapes, 100 + seed, dtype)
        want = X.astype(np.float64) @ kron_all(Fs)
        got = impl(X, Fs)
        assert got.shape == want.shape
        assert np.array_equal(got.astype(np.float64), want), (M, shapes)


def check_vec_trick(impl):
    """N = 2, M = 1: x (A (x) B) = vec_rowmajor(A^T Xmat B) with Xmat = x reshaped to P1 x P2."""
    X, Fs = small_int_problem(1, [(3, 4), (5, 2)], 7)
    A, B = Fs
    want = (A.T @ X.reshape(3, 5) @ B).reshape(1, -1)
    assert np.array_equal(impl(X, Fs), want)


def check_identity(impl, dtype=np.float32):
    X = kron_inputs.draw((3, 4 * 3 * 5), dtype, "uniform", 11, 0)
    Fs = [np.eye(n, dtype=dtype) for n in (4, 3, 5)]
    assert np.array_equal(impl(X, Fs), X)


def check_mixed_product(impl):
    X, AB = small_int_problem(3, [(3, 2), (2, 4)], 21)
    _, CD = small_int_problem(1, [(2, 3), (4, 2)], 22)
    lhs = impl(impl(X, AB), CD)
    rhs = impl(X, [AB[0] @ CD[0], AB[1] @ CD[1]])
    assert np.array_equal(lhs, rhs)


def check_linearity(impl):
    X, Fs = small_int_problem(2, [(2, 3), (3, 3), (4, 2)], 31)
    for i in range(3):
        _, Gs = small_int_problem(1, [(2, 3), (3, 3), (4, 2)], 32 + i)
        mixed = list(Fs)
        mixed[i] = 3 * Fs[i] - 2 * Gs[i]
        other = list(Fs)
        other[i] = Gs[i]
        assert np.array_equal(impl(X, mixed), 3 * impl(X, Fs) - 2 * impl(X, other))


def check_all_ones(impl):
    X, _ = small_int_problem(4, [(4, 4), (2, 2), (3, 3)], 41)
    Fs = [np.ones((4, 5)), np.ones((2, 3)), np.ones((3, 2))]
    Y = impl(X, Fs)
    assert Y.shape == (4, 30)
    assert np.array_equal(Y, np.repeat(X.sum(axis=1, keepdims=True), 30, axis=1))


def check_permutation(impl, dtype=np.float32):
    """Permutation-matrix factors move columns without arithmetic: bit-exact for any float X.
    F_i[p][sigma_i(p)] = 1  =>  Y[:, (sigma_1(p1), sigma_2(p2), ...)] = X[:, (p1, p2, ...)]."""
    sizes = (4, 3, 5)
    rng = np.random.default_rng(5)
    sig = [rng.permutation(n) for n in sizes]
    Fs = []
    for n, s in zip(sizes, sig):
        F = np.zeros((n, n), dtype=dtype)
        F[np.arange(n), s] = 1
        Fs.append(F)
    X = kron_inputs.draw((3, 60), dtype, "uniform", 51, 0)
    want = np.empty_like(X)
    for p1 in range(4):
        for p2 in range(3):
            for p3 in range(5):
                want[:, (sig[0][p1] * 3 + sig[1][p2]) * 5 + sig[2][p3]] = X[:, (p1 * 3 + p2) * 5 + p3]
    assert np.array_equal(impl(X, Fs), want)


def check_rank_one(impl):
    """F_i = u_i v_i^T  =>  Y = (X (x)u_i) (x)v_i^T."""
    rng = np.random.default_rng(6)
    us = [rng.integers(-2, 3, n).astype(np.float64) for n in (3, 4, 2)]
    vs = [rng.integers(-2, 3, n).astype(np.float64) for n in (2, 3, 5)]
    X, _ = small_int_problem(3, [(3, 1), (4, 1), (2, 1)], 61)
    Fs = [np.outer(u, v) for u, v in zip(us, vs)]
    ku = np.kron(np.kron(us[0], us[1]), us[2])
    kv = np.kron(np.kron(vs[0], vs[1]), vs[2])
    assert np.array_equal(impl(X, Fs), np.outer(X @ ku, kv))


def shuffle_algorithm(X, Fs):
    """The reshape / matmul / transpose iteration of section 2.1, as an independent formulation."""
    M = X.shape[0]
    Y = np.asarray(X, dtype=np.float64)
    for F in reversed(Fs):
        P, Q = F.shape
        Y = Y.reshape(-1, P) @ np.asarray(F, dtype=np.float64)     # (a)
        Y = Y.reshape(M, -1, Q).transpose(0, 2, 1)                  # (b)
        Y = Y.reshape(M, -1)                                        # (c)
    return Y


def check_shuffle_equivalence(impl):
    X, Fs = small_int_problem(3, [(4, 2), (3, 3), (2, 5), (2, 2)], 71)
    assert np.array_equal(impl(X, Fs), shuffle_algorithm(X, Fs))


ALL_CHECKS = [check_worked_example, check_against_numpy_kron, check_vec_trick, check_identity,
              check_mixed_product, check_linearity, check_all_ones, check_permutation,
              check_rank_one, check_shuffle_equivalence]


# ---------------------------------------------------------------- the oracle passes every pin

@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda c: c.__name__)
def test_oracle_pin(check):
    check(oracle.kron_matmul)


@pytest.mark.parametrize("check", [check_worked_example, check_against_numpy_kron, check_vec_trick,
                                   check_identity, check_permutation, check_rank_one],
                         ids=lambda c: c.__name__)
def test_bruteforce_pin(check):
    check(oracle.kron_bruteforce)


def test_oracle_f32_io_matches_numpy_kron():
    check_against_numpy_kron(oracle.kron_matmul, np.float32)
    check_against_numpy_kron(oracle.kron_bruteforce, np.float32)


def test_single_iteration_matches_figure():
    g = read_golden("fig2_first_iteration_2x4.txt")
    for dt in (np.float32, np.float64):
        X = np.array(g["x"], dtype=dt).reshape(2, 4)
        F2 = np.array(g["f2"], dtype=dt).reshape(2, 2)
        Y2 = np.array(g["y2"], dtype=dt).reshape(2, 4)
        assert np.array_equal(oracle.sliced_multiply(X, F2), Y2)


def test_single_iterations_chain_to_full_product():
    X, Fs = small_int_problem(3, [(2, 3), (4, 2), (3, 5)], 81)
    Y = X
    for F in reversed(Fs):
        Y = oracle.sliced_multiply(Y, F)
    assert np.array_equal(Y, X @ kron_all(Fs))


def test_random_floats_against_numpy_within_rounding():
    """Float inputs: Algorithm 1 in wide accumulators equals X @ kron within a few ulps."""
    for dt, tol in ((np.float32, 2e-7), (np.float64, 4e-16)):
        X, Fs = kron_inputs.make_problem(5, [(4, 3), (3, 4), (5, 2)], dt, "uniform", "normal", 91)
        want = np.asarray(X, dtype=np.longdouble) @ kron_all(Fs).astype(np.longdouble)
        got = oracle.kron_matmul(X, Fs)
        assert got.dtype == dt
        scale = np.abs(want).max()
        assert np.abs(got - want).max() <= tol * scale * 4


def test_oracle_equals_bruteforce_on_the_small_config():
    X, Fs = kron_inputs.make_config("c1_f32_m16_8x8x3", seed=3)
    a = oracle.kron_matmul(X, Fs)
    b = oracle.kron_bruteforce(X, Fs)
    # both round a wide-precision value once; they may differ by one float32 ulp at most
    assert np.abs(a - b).max() <= np.spacing(np.abs(a).max())
    Xi, Fi = kron_inputs.make_config("c1_f32_m16_8x8x3", seed=3, x="int2", f="int2")
    assert np.array_equal(oracle.kron_matmul(Xi, Fi), oracle.kron_bruteforce(Xi, Fi))


def test_closed_forms_of_cost():
    """Section 3 / section 2.1: iteration i (i = N..1) reads a row of Q^(N-i) P^i columns and writes
    one of Q^(N+1-i) P^(i-1); the elements read add up to M*sum_i Q^(N-i) P^i, and with P = Q the
    multiply-adds are P times that (the paper's computation-to-memory ratio P)."""
    for M, P, Q, N in ((3, 4, 2, 3), (2, 3, 3, 4)):
        K = P ** N
        macs = reads = 0
        for i in range(N, 0, -1):
            assert K == Q ** (N - i) * P ** i
            L = K // P * Q
            assert L == Q ** (N + 1 - i) * P ** (i - 1)
            reads += M * K
            macs += M * L * P
            K = L
        assert reads == M * sum(Q ** (N - i) * P ** i for i in range(1, N + 1))
        if P == Q:
            assert macs == P * reads
        # the oracle's output has the final width
        X = np.zeros((M, P ** N))
        assert oracle.kron_matmul(X, [np.zeros((P, Q))] * N).shape == (M, Q ** N)


def test_invalid_shapes_raise():
    X = np.zeros((2, 6), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.kron_matmul(X, [np.zeros((2, 2), np.float32), np.zeros((2, 2), np.float32)])
    with pytest.raises(ValueError):
        oracle.sliced_multiply(X, np.zeros((4, 2), np.float32))


def test_empty_rows():
    X = np.zeros((0, 4), dtype=np.float64)
    Y = oracle.kron_matmul(X, [np.ones((2, 3)), np.ones((2, 2))])
    assert Y.shape == (0, 6)


# ---------------------------------------------------------------- planted mistakes are caught

def _mutant(kind):
    def impl(X, Fs):
        Fs = [np.asarray(F, dtype=np.float64) for F in Fs]
        M = X.shape[0]
        cur = np.asarray(X, dtype=np.float64)
        order = list(range(len(Fs)))
        seq = order if kind == "first_factor_first" else order[::-1]
        for f in seq:
            F = Fs[f]
            P, Q = F.shape
            K = cur.shape[1]
            S = K // P
            nxt = np.zeros((M, S * Q))
            for j in range(S * Q):
                if kind == "matmul_order":            # consecutive outputs = consecutive columns
                    s, q = j // Q, j % Q
                else:
                    s, q = j % S, j // S
                acc = 0.0
                prange = range(P - 1) if kind == "dropped_term" and P > 1 else range(P)
                for p in prange:
                    if kind == "transposed_factor" and P == Q:
                        acc = acc + cur[:, s * P + p] * F[q, p]
                    elif kind == "strided_slice":     # slice = every S-th element
                        acc = acc + cur[:, p * S + s] * F[p, q]
                    elif kind == "wrong_sign":
                        acc = acc - cur[:, s * P + p] * F[p, q] if p == 1 else acc + cur[:, s * P + p] * F[p, q]
                    else:
                        acc = acc + cur[:, s * P + p] * F[p, q]
                nxt[:, j] = acc
            cur = nxt
        return cur.astype(X.dtype)
    return impl


def test_reference_mutant_is_clean():
    """The un-mutated Python transcription passes every pin (so rejections below are the mistakes')."""
    for check in ALL_CHECKS:
        check(_mutant("none"))


@pytest.mark.parametrize("kind", ["first_factor_first", "matmul_order", "dropped_term",
                                  "transposed_factor", "strided_slice", "wrong_sign"])
def test_pins_catch_planted_mistakes(kind):
    caught = []
    for check in ALL_CHECKS:
        try:
            check(_mutant(kind))
        except (AssertionError, ValueError):
            caught.append(check.__name__)
    assert caught, "no pin rejects the planted mistake %r" % kind
