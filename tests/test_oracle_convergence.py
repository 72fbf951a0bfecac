"""The oracle round drives a decentralised least-squares problem to its optimum (the claim of
Sec. III: consensus and convergence), on synthetic data small enough for the CPU."""
import numpy as np

from oracle import saps_oracle as O


def make_problem(n, N, m, seed):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((n, m, N)).astype(np.float32) / np.sqrt(m)
    x_true = rng.standard_normal(N).astype(np.float32)
    b = np.einsum("imj,j->im", A, x_true) + 0.01 * rng.standard_normal((n, m)).astype(np.float32)
    H = np.einsum("imj,imk->jk", A.astype(np.float64), A.astype(np.float64)) / n
    rhs = np.einsum("imj,im->j", A.astype(np.float64), b.astype(np.float64)) / n
    x_star = np.linalg.solve(H, rhs)                      # minimiser of (1/n) sum_i f_i
    return A, b, x_star


def grads(A, b, X):
    r = np.einsum("imj,ij->im", A, X) - b                # residual of worker i at its own model
    return np.einsum("imj,im->ij", A, r).astype(np.float32)


def test_sparse_gossip_sgd_reaches_the_joint_optimum():
    n, N, m, c, T = 8, 64, 96, 4.0, 400
    A, b, x_star = make_problem(n, N, m, 0)
    rng = np.random.default_rng(1)
    X = rng.standard_normal((n, N)).astype(np.float32)    # workers start apart
    V = np.zeros_like(X)
    _, D0 = O.consensus(X)
    err0 = np.linalg.norm(X.mean(0) - x_star)
    for t in range(1, T + 1):
        perm = rng.permutation(n); peer = np.empty(n, np.int32)
        peer[perm[0::2]] = perm[1::2]; peer[perm[1::2]] = perm[0::2]
        rc, *_ = O.round_(X, grads(A, b, X), V, N, 0.05, 0.9, 11, t, peer, c)
        assert rc == O.OK
    mean, D = O.consensus(X)
    assert np.linalg.norm(mean - x_star) < 0.02 * err0     # the average model found the optimum
    assert D < 1e-3 * D0                                   # and the workers agree (consensus)
