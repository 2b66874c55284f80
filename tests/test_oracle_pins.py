"""The CPU oracle against what the paper and mathematics fix (no GPU)."""
import numpy as np
import pytest

import oracle
from oracle_pins import ALL_CHECKS, check_hand_example


@pytest.fixture(scope="module")
def lib():
    return oracle.load()


@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(lib, check):
    check(lib)


def test_hand_example_f64(lib):
    check_hand_example(lib, dtype="f64")


def test_create_rejects_bad_arguments(lib):
    import numpy as np
    for (W, P, d, tau) in ((0, 4, 1, 1), (2, 4, -1, 1), (2, 4, 1, 0)):
        with pytest.raises((ValueError, AssertionError)):
            oracle.Oracle(W, P, d, tau, 0.1, 0.9, 0.0, np.zeros(max(P, 1)))


# ------------------------------------------------------------------------------------------------
# the matrix form (appendix "Matrix Representation") over randomly drawn tau, d, xi, M: every step of
# the oracle against the recursion written with an explicit history and J as a matrix product
from hypothesis import given, settings, strategies as st


@settings(max_examples=60, deadline=None, derandomize=True)
@given(tau=st.integers(1, 6), d=st.integers(0, 9), xi=st.sampled_from([0.0, 0.125, 0.25, 0.5, 0.75, 1.0]),
       M=st.integers(1, 9), P=st.integers(1, 5), seed=st.integers(0, 2**16))
def test_matrix_form_over_random_schedules(tau, d, xi, M, P, seed):
    import oracle
    r = np.random.default_rng(seed)
    K, eta = 4 * tau + d + 3, 0.05
    J = np.full((M, M), 1.0 / M)
    o = oracle.Oracle(M, P, d, tau, eta, 0.0, 0.0, r.standard_normal(P), xi=xi, dtype="f64")
    Y = []
    for k in range(K):
        G = r.standard_normal((M, P))
        Y.append(o.x.T.copy() - oracle.f32(eta) * G.T)
        o.step(G)
        merge = (k + 1 - d) % tau == 0 and k - d >= tau - 1
        want = oracle.f32(xi) * Y[k] + (1 - oracle.f32(xi)) * (Y[k - d] @ J) if merge else Y[k]
        np.testing.assert_allclose(o.x.T, want, rtol=1e-12, atol=1e-13, err_msg=f"tau={tau} d={d} xi={xi} M={M} k={k}")
    o.close()
