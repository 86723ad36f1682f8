"""Pins of the oracle's greedy binary-coding quantiser (Eq. 1, Sec. II-B) against what the
mathematics fixes: hand-worked examples, the q = 1 optimum by brute force over all sign patterns,
the residual identity, invariances, and exact recovery of matrices that are exactly representable."""
import itertools

import numpy as np
import pytest

from conftest import read_golden


def _examples():
    out = []
    for w, q, alphas, signs in read_golden("eq1_greedy_worked_examples.txt"):
        w = np.array([float(v) for v in w.split(",")], dtype=np.float32)
        alphas = [float(v) for v in alphas.split(",")]
        planes = [[1 if c == "+" else -1 for c in p.strip()] for p in signs.split(";")]
        out.append((w, int(q), alphas, planes))
    return out


def test_worked_examples(oracle):
    for w, q, alphas, planes in _examples():
        B, alpha = oracle.quantize_greedy(w[None, :], q)
        assert alpha[:, 0].tolist() == alphas, (w, alpha)
        assert B[:, 0, :].tolist() == planes, (w, B)


def test_first_plane_is_the_q1_optimum_by_brute_force(oracle):
    """For q = 1 Eq. 1 has a closed-form minimiser once b is fixed (alpha = w.b / n); trying all
    2^n sign patterns gives the global optimum, which the greedy step must reach."""
    rng = np.random.default_rng(11)
    for n in (1, 2, 5, 9):
        for _ in range(5):
            w = rng.standard_normal(n).astype(np.float32)
            best = np.inf
            for signs in itertools.product((-1.0, 1.0), repeat=n):
                b = np.array(signs)
                a = float(w.astype(np.float64) @ b) / n
                best = min(best, float(((w - a * b) ** 2).sum()))
            B, alpha = oracle.quantize_greedy(w[None, :], 1)
            err = float(((w.astype(np.float64) - alpha[0, 0] * B[0, 0]) ** 2).sum())
            assert err <= best * (1 + 1e-12) + 1e-15


def test_every_plane_is_the_q1_optimum_of_its_residual(oracle):
    rng = np.random.default_rng(12)
    w = rng.standard_normal((3, 7)).astype(np.float32)
    B, alpha, R = oracle.quantize_greedy(w, 3, with_residuals=True)
    for i in range(3):
        for r in range(3):
            res = R[i, r]
            best = min(float(((res - (res @ np.array(s)) / 7 * np.array(s)) ** 2).sum())
                       for s in itertools.product((-1.0, 1.0), repeat=7))
            got = float(((res - alpha[i, r] * B[i, r]) ** 2).sum())
            assert got <= best * (1 + 1e-12) + 1e-15


def test_residual_identity_and_monotone_error(oracle):
    """||r_i||^2 = ||r_{i-1}||^2 - n alpha_i^2, hence the reconstruction error never grows with q."""
    rng = np.random.default_rng(13)
    m, n, q = 6, 301, 5
    w = (rng.standard_normal((m, n)) * rng.uniform(0.1, 3.0, size=(m, 1))).astype(np.float32)
    B, alpha, R = oracle.quantize_greedy(w, q, with_residuals=True)
    w64 = w.astype(np.float64)
    assert np.array_equal(R[0], w64)
    prev = (w64 ** 2).sum(axis=1)
    for i in range(q):
        rec = np.einsum("im,imn->mn", alpha[: i + 1], B[: i + 1].astype(np.float64))
        err = ((w64 - rec) ** 2).sum(axis=1)
        np.testing.assert_allclose(err, prev - n * alpha[i] ** 2, rtol=1e-9, atol=1e-12)
        assert np.all(err <= prev + 1e-12)
        if i + 1 < q:
            np.testing.assert_allclose(R[i + 1], w64 - rec, rtol=0, atol=1e-12)
        prev = err
    # closed forms of the first plane
    np.testing.assert_allclose(alpha[0], np.abs(w64).mean(axis=1), rtol=1e-14)
    assert np.array_equal(B[0], np.where(w64 < 0, -1, 1))


def test_invariances(oracle):
    rng = np.random.default_rng(14)
    w = rng.standard_normal((4, 64)).astype(np.float32)
    B, alpha = oracle.quantize_greedy(w, 3)
    B2, alpha2 = oracle.quantize_greedy(w * np.float32(4.0), 3)   # exact scaling by a power of two
    assert np.array_equal(B, B2) and np.array_equal(alpha * 4.0, alpha2)
    perm = rng.permutation(64)
    B3, alpha3 = oracle.quantize_greedy(w[:, perm], 3)            # element order does not matter
    assert np.array_equal(B[:, :, perm], B3)
    np.testing.assert_allclose(alpha3, alpha, rtol=1e-13)
    B4, alpha4 = oracle.quantize_greedy(w[::-1].copy(), 3)        # rows are independent
    assert np.array_equal(B[:, ::-1], B4) and np.array_equal(alpha[:, ::-1], alpha4)


def test_exactly_representable_rows_are_recovered(oracle):
    """w = a1 b1 + a2 b2 with a1 > a2 > 0 and b1.b2 = 0 (balanced agreement): the greedy steps
    find a1, b1, a2, b2 exactly and leave no residual."""
    b1 = np.array([1, 1, 1, 1, -1, -1, -1, -1], dtype=np.float64)
    b2 = np.array([1, 1, -1, -1, 1, 1, -1, -1], dtype=np.float64)
    w = (0.75 * b1 + 0.25 * b2).astype(np.float32)
    B, alpha, R = oracle.quantize_greedy(w[None, :], 3, with_residuals=True)
    assert alpha[:, 0].tolist() == [0.75, 0.25, 0.0]
    assert np.array_equal(B[0, 0], b1) and np.array_equal(B[1, 0], b2)
    assert np.all(R[2] == 0.0)


def test_zero_of_either_sign_takes_plus_one(oracle):
    """Eq. 1 with sign(0) = +1: a weight that is +0.0 or -0.0 (a pruned weight computed as
    negative * 0) gets b = +1, and its residual continues as 0 - alpha.  Hand-worked row
    w = (-0, +0, 4, -4): alpha_1 = 2, b_1 = (+,+,+,-), r = (-2,-2,2,-2), alpha_2 = 2, b_2 = (-,-,+,-)."""
    w = np.array([[-0.0, 0.0, 4.0, -4.0]], dtype=np.float32)
    assert np.signbit(w[0, 0]) and not np.signbit(w[0, 1])
    B, alpha, R = oracle.quantize_greedy(w, 2, with_residuals=True)
    assert alpha[:, 0].tolist() == [2.0, 2.0]
    assert B[0, 0].tolist() == [1, 1, 1, -1]
    assert R[1, 0].tolist() == [-2.0, -2.0, 2.0, -2.0]
    assert B[1, 0].tolist() == [-1, -1, 1, -1]


def test_argument_errors(oracle):
    with pytest.raises(oracle.OracleError):
        oracle.quantize_greedy(np.zeros((2, 3), np.float32), 0)
