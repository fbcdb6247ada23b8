"""The library's host-side policy search (Algorithm 1) and similarity matrix, called through
the C ABI, against the oracle and against exhaustive search.  No GPU is needed: these two
entry points take host arrays and launch nothing."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2602_00777_amd import binding


def value_of(M, policy, theta):
    src, C, S = 0, 0, 0.0
    for j, a in enumerate(policy):
        if a == 0:
            src, C = j, C + 1
        elif M[src, j] < theta:
            return None
        S += M[src, j]
    return C, S


@pytest.mark.parametrize("seed", range(6))
def test_policy_search_matches_oracle_and_exhaustive_search(seed):
    rng = np.random.RandomState(100 + seed)
    L = 5 + seed
    M = np.triu(rng.uniform(0.1, 1.0, size=(L, L)))
    np.fill_diagonal(M, 1.0)
    for theta in (0.0, 0.3, 0.6, 0.9, 1.0):
        pol, C, S = binding.policy_search(M, theta)
        opol, oC, oS = oracle.policy_search(M, theta)
        assert pol.tolist() == opol.tolist() and C == oC and S == oS
        best = None
        for bits in itertools.product((0, 1), repeat=L - 1):
            v = value_of(M, (0,) + bits, theta)
            if v is not None and (best is None or v[0] < best[0] or (v[0] == best[0] and v[1] > best[1])):
                best = v
        assert (C, pytest.approx(S, abs=1e-12)) == best


def test_policy_search_with_ties_matches_oracle():
    """Quantised similarities (many equal path values): the tie rule must be the oracle's."""
    rng = np.random.RandomState(7)
    for L in (6, 9, 13, 32):
        M = np.triu(rng.randint(0, 4, size=(L, L)) / 4.0)
        np.fill_diagonal(M, 1.0)
        for theta in (0.25, 0.5, 0.75):
            pol, C, S = binding.policy_search(M, theta)
            opol, oC, oS = oracle.policy_search(M, theta)
            assert pol.tolist() == opol.tolist() and C == oC and S == oS
            assert value_of(M, pol, theta) == (C, pytest.approx(S))


def test_similarity_matrix_from_counts():
    counts = np.array([[8, 4, 2], [0, 8, 6], [0, 0, 4]], np.int64)
    M = binding.similarity_matrix(counts)
    assert M.tolist() == [[1.0, 0.5, 0.5], [0.0, 1.0, 1.5], [0.0, 0.0, 1.0]]
    assert np.array_equal(M, oracle.similarity_matrix(counts))
    empty = np.array([[8, 0], [0, 0]], np.int64)          # a layer without valid entries
    assert binding.similarity_matrix(empty).tolist() == [[1.0, 0.0], [0.0, 1.0]]


def test_policy_search_argument_errors():
    lib = binding.load_library()
    M = np.eye(3)
    pol = np.empty(3, np.uint8)
    assert lib.hylra_policy_search(None, 0, M.ctypes.data, 0.5, pol.ctypes.data, None, None) == 1
    assert lib.hylra_policy_search(None, 3, None, 0.5, pol.ctypes.data, None, None) == 1
    assert lib.hylra_policy_search(None, 3, M.ctypes.data, float("nan"), pol.ctypes.data, None, None) == 1
    assert lib.hylra_similarity_matrix(3, None, M.ctypes.data) == 1
