"""Property tests of the oracle round over random small shapes (hypothesis): the invariants that
Sec. II-B/II-C and Sec. III fix must hold for every shape, ratio, matching, seed and round."""
import numpy as np
import pytest

hyp = pytest.importorskip("hypothesis")
from hypothesis import given, settings, strategies as st   # noqa: E402

import independent_philox as IP                              # noqa: E402
from oracle import saps_oracle as O                          # noqa: E402


@st.composite
def cases(draw):
    n = draw(st.integers(1, 7))
    N = draw(st.integers(1, 300))
    c = draw(st.sampled_from([1, 2, 3, 5, 10, 100]))
    seed = draw(st.integers(0, 2**64 - 1))
    rnd = draw(st.integers(0, 2**64 - 1))
    perm = draw(st.permutations(list(range(n))))
    singles = draw(st.integers(0, n))
    peer = np.arange(n, dtype=np.int32)
    rest = list(perm)[singles:]
    for a in range(0, len(rest) - 1, 2):
        peer[rest[a]], peer[rest[a + 1]] = rest[a + 1], rest[a]
    data_seed = draw(st.integers(0, 2**31))
    return n, N, c, seed, rnd, peer, data_seed


@settings(max_examples=150, deadline=None)
@given(cases())
def test_exchange_invariants(case):
    n, N, c, seed, rnd, peer, data_seed = case
    rng = np.random.default_rng(data_seed)
    X0 = rng.integers(-512, 512, (n, N)).astype(np.float32) / 8.0       # exact halves, exact sums
    X = X0.copy()
    rc, K, idx, msg = O.round_(X, None, None, N, 0, 0, seed, rnd, peer, float(c))
    assert rc == O.OK
    keep = np.array([IP.keep(seed, rnd, j, c) for j in range(N)], dtype=bool)
    assert K == int(keep.sum()) and np.array_equal(idx[:K], np.flatnonzero(keep).astype(np.uint32))
    assert np.array_equal(msg[:, :K], X0[:, keep])
    assert np.array_equal(X[:, ~keep], X0[:, ~keep])                     # Eq. (7): X o notM untouched
    for i in range(n):
        p = int(peer[i])
        if p == i:
            assert np.array_equal(X[i], X0[i])                           # unmatched worker keeps its model
        else:
            assert np.array_equal(X[i, keep], (X0[i, keep] + X0[p, keep]) / 2)   # GenerateW: weights 1/2, 1/2
            assert np.array_equal(X[i, keep], X[p, keep])
    assert np.array_equal(X.sum(0), X0.sum(0))                           # W doubly stochastic: column sums kept
    _, D0 = O.consensus(X0); _, D1 = O.consensus(X)
    assert D1 <= D0 * (1 + 1e-12) + 1e-12                                # averaging never increases disagreement


@settings(max_examples=80, deadline=None)
@given(cases(), st.floats(0.0, 0.5), st.floats(0.0, 0.95), st.booleans())
def test_round_is_step_then_exchange_or_exchange_then_step(case, lr, mu, mix_first):
    n, N, c, seed, rnd, peer, data_seed = case
    rng = np.random.default_rng(data_seed)
    X0 = rng.standard_normal((n, N)).astype(np.float32); G = rng.standard_normal((n, N)).astype(np.float32)
    V0 = rng.standard_normal((n, N)).astype(np.float32)
    X, V = X0.copy(), V0.copy()
    rc, K, idx, msg = O.round_(X, G, V, N, lr, mu, seed, rnd, peer, float(c), mix_first=mix_first)
    assert rc == O.OK
    # the same result from the single-stage entries in the stated order
    Y, W = X0.copy(), V0.copy()
    if not mix_first:
        O.sgd_step(Y, G, W, lr, mu)
    rc2, K2, idx2, msg2 = O.mask_compact(Y, N, seed, rnd, float(c))
    assert (rc2, K2) == (O.OK, K)
    O.merge(Y, N, peer, idx2, msg2, K2)
    if mix_first:
        O.sgd_step(Y, G, W, lr, mu)
    assert np.array_equal(X.view(np.uint32), Y.view(np.uint32)) and np.array_equal(V.view(np.uint32), W.view(np.uint32))
    assert np.array_equal(msg[:, :K].view(np.uint32), msg2[:, :K].view(np.uint32))
