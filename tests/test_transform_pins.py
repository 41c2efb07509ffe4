"""CPU pins of the oracle's online activation transform X <- X . D . (P1 kron P2) (section "Learnable
Transformation": transformation pair T = D P with a Kronecker-factored P; "Integration into Transformer
Architecture": Y = X W^T = (X T)(T^-1 W^T)).  Each pin checks the oracle against something it does not
compute itself: numpy's Kronecker product, the two-sided matrix form, special cases, the paper's inverse and
reparameterisation identities."""
import numpy as np
import pytest

import btc_synth as S


def _x(rng, M, n, kind="f16"):
    return S.draw_x(rng, M, n, kind)


def _sigma(bits, n):
    k = np.arange(n)
    return np.where((bits[k >> 5] >> (k & 31).astype(np.uint32)) & 1, 1.0, -1.0)


@pytest.mark.parametrize("n1,n2,M,kind", [(3, 5, 4, "f16"), (8, 4, 2, "bf16"), (7, 7, 3, "f16"), (1, 9, 2, "f16"),
                                           (6, 1, 2, "bf16")])
def test_against_numpy_kron(oracle, n1, n2, M, kind):
    bits, P1, P2 = S.draw_transform(3, n1, n2)
    rng = np.random.default_rng(5)
    xb = _x(rng, M, n1 * n2, kind)
    X = oracle.widen(xb, kind)
    T = _sigma(bits, n1 * n2)[:, None] * np.kron(P1.astype(np.float64), P2.astype(np.float64))
    np.testing.assert_allclose(oracle.transform(xb, bits, P1, P2, kind), X @ T, rtol=1e-12, atol=1e-13)


def test_two_sided_form(oracle):
    """Row m, reshaped to n1 x n2, becomes P1^T (X_m sigma) P2: a transposed factor or a swapped pair fails."""
    n1, n2, M = 12, 10, 3
    bits, P1, P2 = S.draw_transform(11, n1, n2)
    rng = np.random.default_rng(2)
    xb = _x(rng, M, n1 * n2)
    X = oracle.widen(xb, "f16") * _sigma(bits, n1 * n2)
    want = np.stack([(P1.astype(np.float64).T @ X[m].reshape(n1, n2) @ P2.astype(np.float64)).reshape(-1)
                     for m in range(M)])
    np.testing.assert_allclose(oracle.transform(xb, bits, P1, P2), want, rtol=1e-12, atol=1e-13)


def test_identity_factors_give_sign_flips(oracle):
    n1, n2 = 4, 6
    bits, _, _ = S.draw_transform(1, n1, n2)
    rng = np.random.default_rng(0)
    xb = _x(rng, 2, n1 * n2)
    got = oracle.transform(xb, bits, np.eye(n1, dtype=np.float32), np.eye(n2, dtype=np.float32))
    assert np.array_equal(got, oracle.widen(xb, "f16") * _sigma(bits, n1 * n2))


def test_unit_vector_reads_one_row_of_T(oracle):
    """x = e_i picks row i of T: sigma_i * P1[i1][:] kron P2[i2][:] (exact products of two fp32 numbers)."""
    n1, n2 = 5, 3
    bits, P1, P2 = S.draw_transform(9, n1, n2)
    sig = _sigma(bits, n1 * n2)
    for i in (0, 4, 7, 14):
        x = np.zeros((1, n1 * n2), dtype=np.float16)
        x[0, i] = 1.0
        got = oracle.transform(x.view(np.uint16), bits, P1, P2)[0]
        i1, i2 = divmod(i, n2)
        want = sig[i] * np.outer(P1[i1].astype(np.float64), P2[i2].astype(np.float64)).reshape(-1)
        assert np.array_equal(got, want)


def test_inverse_is_kronecker_of_inverses(oracle):
    """P^-1 = P1^-1 kron P2^-1: with all signs +1, transforming by (P1, P2) and then by the inverses (rounded to
    fp32, hence the tolerance) returns the input."""
    n1, n2 = 8, 6
    _, P1, P2 = S.draw_transform(4, n1, n2)
    plus = np.full(((n1 * n2 + 31) // 32,), 0xFFFFFFFF, dtype=np.uint32)
    rng = np.random.default_rng(1)
    xb = _x(rng, 3, n1 * n2)
    X = oracle.widen(xb, "f16")
    Y = oracle.transform(xb, plus, P1, P2)
    Pi = np.kron(np.linalg.inv(P1.astype(np.float64)), np.linalg.inv(P2.astype(np.float64)))
    np.testing.assert_allclose(Y @ Pi, X, rtol=0, atol=1e-10)


def test_layer_output_is_unchanged_by_the_pair(oracle):
    """Y = X W^T = (X T)(T^-1 W^T): the transform multiplies activations from the right."""
    n1, n2, out = 6, 5, 7
    bits, P1, P2 = S.draw_transform(6, n1, n2)
    rng = np.random.default_rng(3)
    xb = _x(rng, 4, n1 * n2)
    X = oracle.widen(xb, "f16")
    W = rng.standard_normal((out, n1 * n2))
    T = _sigma(bits, n1 * n2)[:, None] * np.kron(P1.astype(np.float64), P2.astype(np.float64))
    XT = oracle.transform(xb, bits, P1, P2)
    np.testing.assert_allclose(XT @ (np.linalg.inv(T) @ W.T), X @ W.T, rtol=0, atol=1e-9)


def test_rows_are_independent_and_linear(oracle):
    n1, n2 = 4, 8
    bits, P1, P2 = S.draw_transform(8, n1, n2)
    a = np.arange(n1 * n2, dtype=np.float16).reshape(1, -1) - 10
    b = ((np.arange(n1 * n2) * 7) % 13).astype(np.float16).reshape(1, -1)
    both = np.concatenate([a, b, (2 * a + b).astype(np.float16)])          # small integers: exact in fp16
    Y = oracle.transform(both.view(np.uint16), bits, P1, P2)
    np.testing.assert_allclose(Y[2], 2 * Y[0] + Y[1], rtol=1e-13, atol=1e-12)
    assert np.array_equal(Y[0], oracle.transform(a.view(np.uint16), bits, P1, P2)[0])
