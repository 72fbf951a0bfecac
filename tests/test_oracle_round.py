"""Pins of the oracle's update, compaction, merge and round — CPU only.

Nothing here re-calls the oracle to check the oracle: expected values come from the
explicit matrices of Eq. (7), from numpy/torch library routines, from closed forms, or
from invariants the paper states (doubly stochastic W, Lemma 1, Lemma 2).
"""
import itertools

import numpy as np
import pytest

import independent_philox as IP
from oracle import saps_oracle as O


def _mask_indep(N, seed, rnd, c):
    return np.array([IP.keep(seed, rnd, j, c) for j in range(N)], dtype=bool)


def _W(peer):
    """GenerateW of Alg. 3 for a matching; an unmatched worker keeps weight 1 on itself."""
    n = len(peer)
    W = np.zeros((n, n))
    for i, p in enumerate(peer):
        if p == i:
            W[i, i] = 1.0
        else:
            W[i, i] = 0.5
            W[i, p] = 0.5
    return W


def _matchings4():
    return [[1, 0, 3, 2], [2, 3, 0, 1], [3, 2, 1, 0], [0, 1, 2, 3], [1, 0, 2, 3], [0, 3, 2, 1]]


# ---------------------------------------------------------------- brute force, Eq. (7)
@pytest.mark.parametrize("n,N", [(2, 1), (2, 7), (3, 13), (4, 64), (4, 61)])
@pytest.mark.parametrize("c", [1, 2, 4])
def test_exchange_equals_explicit_matrix_form(n, N, c):
    rng = np.random.default_rng(n * 1000 + N * 10 + c)
    if n == 4:
        peers = _matchings4()
    elif n == 3:
        peers = [[1, 0, 2], [0, 2, 1], [2, 1, 0], [0, 1, 2]]
    else:
        peers = [[1, 0], [0, 1]]
    for rnd, peer in enumerate(peers, start=1):
        X = rng.standard_normal((n, N)).astype(np.float32)
        m = _mask_indep(N, 42, rnd, c)
        # paper orientation: columns are workers (N x n); M has identical columns
        Xp = X.T.astype(np.float64)
        M = np.repeat(m[:, None], n, axis=1).astype(np.float64)
        want = (Xp * (1 - M) + (Xp * M) @ _W(peer)).T.astype(np.float32)
        got = X.copy()
        rc, K, idx, msg = O.round_(got, None, None, N, 0.0, 0.0, 42, rnd, np.array(peer), float(c))
        assert rc == O.OK
        assert K == int(m.sum())
        assert np.array_equal(idx[:K], np.flatnonzero(m).astype(np.uint32))
        assert np.array_equal(msg[:, :K], X[:, m])
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_round_with_update_equals_matrix_form_after_local_step():
    # Alg. 2 order: local step first, then the exchange of the updated models.
    n, N, c = 4, 64, 2
    rng = np.random.default_rng(77)
    X = rng.standard_normal((n, N)).astype(np.float32)
    G = rng.standard_normal((n, N)).astype(np.float32)
    lr = np.float32(0.25)
    peer = [2, 3, 0, 1]
    m = _mask_indep(N, 1, 1, c)
    # plain SGD (mu = 0, no buffer): x - lr*g with a single rounding = exact product in double, one rounding to fp32
    Xu = (X.astype(np.float64) - np.float64(lr) * G.astype(np.float64)).astype(np.float32)
    Xp = Xu.T.astype(np.float64)
    M = np.repeat(m[:, None], n, axis=1).astype(np.float64)
    want = (Xp * (1 - M) + (Xp * M) @ _W(peer)).T.astype(np.float32)
    got = X.copy()
    rc, K, idx, msg = O.round_(got, G, None, N, float(lr), 0.0, 1, 1, np.array(peer), float(c))
    assert rc == O.OK
    assert np.array_equal(msg[:, :K], Xu[:, m])        # the message carries post-update values
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


# ---------------------------------------------------------------------- local update
def test_update_matches_torch_sgd_momentum():
    torch = pytest.importorskip("torch")
    n, N, steps = 3, 1000, 6
    rng = np.random.default_rng(3)
    X = (0.05 * rng.standard_normal((n, N))).astype(np.float32)
    V = np.zeros_like(X)
    params = [torch.nn.Parameter(torch.from_numpy(X[i].copy())) for i in range(n)]
    opt = torch.optim.SGD(params, lr=0.1, momentum=0.9)
    for t in range(steps):
        G = (1e-3 * rng.standard_normal((n, N))).astype(np.float32)
        for i in range(n):
            params[i].grad = torch.from_numpy(G[i].copy())
        opt.step()
        assert O.sgd_step(X, G, V, 0.1, 0.9) == O.OK
    ref = np.stack([p.detach().numpy() for p in params])
    np.testing.assert_allclose(X, ref, rtol=1e-6, atol=1e-9)


def test_update_is_two_fused_multiply_adds():
    # Reading fixed by this build: v = fma(mu, v, g); x = fma(-lr, v, x), each rounded once.
    rng = np.random.default_rng(8)
    x = rng.standard_normal((1, 4096)).astype(np.float32)
    g = rng.standard_normal((1, 4096)).astype(np.float32)
    v = rng.standard_normal((1, 4096)).astype(np.float32)
    lr, mu = np.float32(0.3), np.float32(0.7)
    # exact products in float64 (24x24-bit mantissas fit), one rounding per fma
    v_ref = (np.float64(mu) * v.astype(np.float64) + g.astype(np.float64)).astype(np.float32)
    x_ref = (x.astype(np.float64) - np.float64(lr) * v_ref.astype(np.float64)).astype(np.float32)
    X, V = x.copy(), v.copy()
    O.sgd_step(X, g, V, float(lr), float(mu))
    # double rounding through float64 can differ from a true fma only on exact ties in the
    # 29 guard bits; none occur for these draws, so equality is bitwise
    assert np.array_equal(V, v_ref)
    assert np.array_equal(X, x_ref)


def test_update_without_buffer_and_padding_untouched():
    n, N, ld = 2, 10, 16
    X = np.full((n, ld), 7.0, np.float32); G = np.full((n, ld), 1.0, np.float32)
    assert O.sgd_step(X, G, None, 0.5, 0.0, N=N) == O.OK
    assert np.all(X[:, :N] == 6.5) and np.all(X[:, N:] == 7.0)
    assert O.sgd_step(X, G, None, 0.5, 0.9, N=N) == O.EINVAL        # momentum needs a buffer


def test_identity_matching_is_pure_update():
    n, N = 4, 500
    rng = np.random.default_rng(0)
    X = rng.standard_normal((n, N)).astype(np.float32); G = rng.standard_normal((n, N)).astype(np.float32)
    V = rng.standard_normal((n, N)).astype(np.float32)
    X2, V2 = X.copy(), V.copy()
    O.sgd_step(X2, G, V2, 0.1, 0.9)
    rc, K, idx, msg = O.round_(X, G, V, N, 0.1, 0.9, 3, 1, np.arange(n), 4.0)
    assert rc == O.OK and np.array_equal(X, X2) and np.array_equal(V, V2)
    assert np.array_equal(msg[:, :K], X2[:, idx[:K]])


# -------------------------------------------------------------------------- compaction
def test_compaction_c1_is_a_row_copy():
    n, N, ld = 3, 257, 260
    rng = np.random.default_rng(1)
    X = rng.standard_normal((n, ld)).astype(np.float32)
    rc, K, idx, msg = O.mask_compact(X, N, 5, 9, 1.0)
    assert rc == O.OK and K == N
    assert np.array_equal(idx, np.arange(N, dtype=np.uint32))
    assert np.array_equal(msg, X[:, :N])


def test_compaction_is_stable_and_complete():
    n, N = 2, 50_000
    rng = np.random.default_rng(2)
    X = rng.standard_normal((n, N)).astype(np.float32)
    rc, K, idx, msg = O.mask_compact(X, N, 17, 3, 100.0)
    assert rc == O.OK
    keep = O.mask(N, 17, 3, 100.0)
    assert K == keep.sum()
    assert np.all(np.diff(idx[:K].astype(np.int64)) > 0)
    assert keep[idx[:K]].all()
    assert np.array_equal(msg[:, :K].view(np.uint32), X[:, idx[:K]].view(np.uint32))


def test_capacity_error_writes_nothing():
    n, N = 2, 4000
    X = np.ones((n, N), np.float32)
    rc, K, idx, msg = O.mask_compact(X, N, 0, 1, 2.0, msg_ld=100)
    assert rc == O.ECAPACITY and K > 100
    assert not idx.any() and not msg.any()
    X0 = X.copy(); G = np.ones_like(X); V = np.zeros_like(X)
    rc, K, idx, msg = O.round_(X, G, V, N, 0.1, 0.9, 0, 1, np.array([1, 0]), 2.0, msg_ld=100)
    assert rc == O.ECAPACITY and np.array_equal(X, X0) and not V.any() and not msg.any()


# ------------------------------------------------------------------------------- merge
def test_merge_invariants_pair_sum_symmetry_idempotence():
    n, N, c = 6, 20_000, 10.0
    rng = np.random.default_rng(4)
    X0 = (0.05 * rng.standard_normal((n, N))).astype(np.float32)
    peer = np.array([3, 4, 5, 0, 1, 2])
    X = X0.copy()
    rc, K, idx, msg = O.round_(X, None, None, N, 0, 0, 9, 1, peer, c)
    m = np.zeros(N, bool); m[idx[:K]] = True
    # unmasked coordinates untouched, bit for bit
    assert np.array_equal(X[:, ~m].view(np.uint32), X0[:, ~m].view(np.uint32))
    for i in range(3):
        a, b = X0[i, m], X0[peer[i], m]
        # both peers hold the same bits and they are the single-rounding mean
        assert np.array_equal(X[i, m].view(np.uint32), X[peer[i], m].view(np.uint32))
        assert np.array_equal(X[i, m], ((a.astype(np.float64) + b.astype(np.float64)) / 2).astype(np.float32))
        # pair sum preserved: out_i + out_p == fl(a + b)
        assert np.array_equal(X[i, m] + X[peer[i], m], a + b)
    # column sums (mean model) preserved: W doubly stochastic
    np.testing.assert_allclose(X.astype(np.float64).sum(0), X0.astype(np.float64).sum(0), rtol=0, atol=n * 2.0**-24)
    # same mask and matching again changes nothing (W^2 = W on the masked block)
    X2 = X.copy()
    O.round_(X2, None, None, N, 0, 0, 9, 1, peer, c)
    assert np.array_equal(X2.view(np.uint32), X.view(np.uint32))


def test_lemma1_mask_and_mix_commute():
    # (A o M) W == (A W) o M when M has identical columns: the sparse exchange equals the dense
    # one on masked coordinates and the identity elsewhere.
    n, N = 4, 5000
    rng = np.random.default_rng(6)
    A = rng.standard_normal((n, N)).astype(np.float32)
    peer = np.array([1, 0, 3, 2])
    Y = A.copy(); Z = A.copy()
    _, K, idx, _ = O.round_(Y, None, None, N, 0, 0, 2, 5, peer, 4.0)
    O.round_(Z, None, None, N, 0, 0, 2, 5, peer, 1.0)          # c = 1: dense gossip step A W
    AW = (A.T.astype(np.float64) @ _W(peer)).T.astype(np.float32)
    assert np.array_equal(Z, AW)
    m = np.zeros(N, bool); m[idx[:K]] = True
    assert np.array_equal(Y[:, m], AW[:, m]) and np.array_equal(Y[:, ~m], A[:, ~m])


def test_c1_fixed_matching_makes_pairs_identical_every_round():
    n, N = 4, 3000
    rng = np.random.default_rng(10)
    X = rng.standard_normal((n, N)).astype(np.float32); V = np.zeros_like(X)
    peer = np.array([2, 3, 0, 1])
    for t in range(1, 5):
        G = rng.standard_normal((n, N)).astype(np.float32)
        rc, K, _, _ = O.round_(X, G, V, N, 0.1, 0.9, 1, t, peer, 1.0)
        assert rc == O.OK and K == N
        assert np.array_equal(X[0].view(np.uint32), X[2].view(np.uint32))
        assert np.array_equal(X[1].view(np.uint32), X[3].view(np.uint32))
        assert not np.array_equal(X[0], X[1])


def test_merge_rejects_bad_matchings():
    X = np.zeros((3, 8), np.float32)
    for bad in ([1, 2, 0], [0, 1, 3], [-1, 1, 2], [1, 1, 2]):
        rc, *_ = O.round_(X, None, None, 8, 0, 0, 0, 1, np.array(bad), 2.0)
        assert rc == O.EMATCH


def test_merge_special_values():
    N = 8
    inf, nan = np.float32(np.inf), np.float32(np.nan)
    tiny = np.float32(1e-45)                               # smallest subnormal
    a = np.array([inf, inf, nan, -0.0, tiny, 3 * tiny, 3.4e38, 1.0], np.float32)
    b = np.array([1.0, -inf, 1.0, 0.0, tiny, tiny, 3.4e38, -1.0], np.float32)
    X = np.stack([a, b])
    O.round_(X, None, None, N, 0, 0, 0, 1, np.array([1, 0]), 1.0)
    with np.errstate(all="ignore"):
        ref = (a + b) * np.float32(0.5)
    assert np.array_equal(np.isnan(X[0]), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(X[0][ok].view(np.uint32), ref[ok].view(np.uint32))
    assert np.array_equal(X[1][ok].view(np.uint32), ref[ok].view(np.uint32))
    assert X[0][0] == inf and np.isnan(X[0][1]) and X[0][4] == tiny and X[0][5] == 2 * tiny and X[0][6] == inf
    assert X[0][3] == 0 and not np.signbit(X[0][3])         # (-0) + (+0) = +0


# ------------------------------------------------------------- multi-round statistics
def test_sparse_gossip_contraction_rate_and_mean_preservation():
    # Lemma 2 with W = (I+P)/2 a projection: per-round expected disagreement ratio is q + p*rho,
    # rho = (n-2)/(2(n-1)) for uniformly random perfect matchings.
    n, N, c, T = 8, 40_000, 4.0, 12
    rng = np.random.default_rng(12)
    X = rng.standard_normal((n, N)).astype(np.float32)
    mean0 = X.astype(np.float64).mean(0)
    D0 = ((X - mean0) ** 2).sum()
    for t in range(1, T + 1):
        perm = rng.permutation(n); peer = np.empty(n, np.int32)
        peer[perm[0::2]] = perm[1::2]; peer[perm[1::2]] = perm[0::2]
        rc, *_ = O.round_(X, None, None, N, 0, 0, 99, t, peer, c)
        assert rc == O.OK
    meanT = X.astype(np.float64).mean(0)
    DT = ((X - meanT) ** 2).sum()
    p, q, rho = 1 / c, 1 - 1 / c, (n - 2) / (2 * (n - 1))
    assert abs(DT / D0 / (q + p * rho) ** T - 1) < 0.03
    # the printed rate with rho^2 is measurably different, so this test tells the readings apart
    assert abs(DT / D0 / (q + p * rho**2) ** T - 1) > 0.15
    np.testing.assert_allclose(meanT, mean0, atol=1e-6)


def test_expected_traffic_matches_2N_over_c():
    # Sec. II-D: per round a worker sends and receives N/c values.
    N, c = 272_474, 100.0
    Ks = [int(O.mask(N, 0, t, c).sum()) for t in range(1, 21)]
    assert abs(np.mean(Ks) - N / c) < 5 * np.sqrt(N / c / 20)


# ------------------------------------------------------------------ consensus diagnostics
def test_consensus_matches_numpy_and_closed_forms():
    rng = np.random.default_rng(21)
    n, N, ld = 7, 3001, 3008
    X = np.full((n, ld), 1e9, np.float32)                  # padding must be ignored
    X[:, :N] = rng.standard_normal((n, N)).astype(np.float32)
    mean, D = O.consensus(X, N)
    X64 = X[:, :N].astype(np.float64)
    assert np.array_equal(mean, X64.mean(0).astype(np.float32))
    assert abs(D - ((X64 - X64.mean(0)) ** 2).sum()) <= 1e-12 * D
    # identical rows: zero disagreement
    Y = np.repeat(X[:1], n, axis=0).copy()
    assert O.consensus(Y, N)[1] == 0.0
    # rows a + i*b (exact in fp32): D = sum_j b_j^2 * sum_i (i - (n-1)/2)^2
    a = rng.integers(-8, 8, N).astype(np.float32); b = rng.integers(-4, 4, N).astype(np.float32)
    Z = np.stack([a + i * b for i in range(n)]).astype(np.float32)
    want = float((b.astype(np.float64) ** 2).sum() * sum((i - (n - 1) / 2) ** 2 for i in range(n)))
    m, D = O.consensus(np.ascontiguousarray(Z))
    assert D == want and np.array_equal(m, (a + (n - 1) / 2 * b).astype(np.float32))


def test_dense_pair_averaging_lowers_disagreement_by_half_the_pair_distances():
    # For W = (I + P)/2:  D(XW) = D(X) - 1/2 * sum over pairs ||x_i - x_p||^2, and the mean is unchanged.
    n, N = 6, 4000
    rng = np.random.default_rng(22)
    X = rng.integers(-64, 64, (n, N)).astype(np.float32)     # small integers: averaging is exact
    peer = np.array([1, 0, 4, 5, 2, 3])
    m0, D0 = O.consensus(X)
    pair = sum(float(((X[i].astype(np.float64) - X[p]) ** 2).sum()) for i, p in enumerate(peer) if p > i)
    O.round_(X, None, None, N, 0, 0, 3, 1, peer, 1.0)
    m1, D1 = O.consensus(X)
    assert np.array_equal(m0, m1)
    assert abs(D1 - (D0 - 0.5 * pair)) <= 1e-12 * D0


# ------------------------------------------------------------------- Eq. (7) ordering
@pytest.mark.parametrize("c", [1, 2, 4])
def test_mix_then_step_order_equals_explicit_matrix_form_with_gradient_term(c):
    # X_{t+1} = X o notM + (X o M) W - gamma G(X_t), plain SGD (no momentum buffer)
    n, N = 4, 64
    rng = np.random.default_rng(31 + c)
    lr = np.float32(0.125)
    for rnd, peer in enumerate(_matchings4(), start=1):
        X = rng.standard_normal((n, N)).astype(np.float32)
        G = rng.standard_normal((n, N)).astype(np.float32)
        m = _mask_indep(N, 5, rnd, c)
        Xp = X.T.astype(np.float64)
        M = np.repeat(m[:, None], n, axis=1).astype(np.float64)
        mixed = (Xp * (1 - M) + (Xp * M) @ _W(peer)).T.astype(np.float32)          # exact halves, one rounding
        want = (mixed.astype(np.float64) - np.float64(lr) * G.astype(np.float64)).astype(np.float32)
        got = X.copy()
        rc, K, idx, msg = O.round_(got, G, None, N, float(lr), 0.0, 5, rnd, np.array(peer), float(c), mix_first=True)
        assert rc == O.OK and K == int(m.sum())
        assert np.array_equal(msg[:, :K], X[:, m])                                  # messages carry X_t
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_mix_then_step_and_alg2_orders_differ_only_on_masked_coordinates_of_matched_rows():
    n, N = 4, 2000
    rng = np.random.default_rng(40)
    X = rng.standard_normal((n, N)).astype(np.float32); G = rng.standard_normal((n, N)).astype(np.float32)
    V = rng.standard_normal((n, N)).astype(np.float32)
    peer = np.array([1, 0, 2, 3])                                                  # rows 2, 3 unmatched
    A, VA, Bm, VB = X.copy(), V.copy(), X.copy(), V.copy()
    _, K, idx, _ = O.round_(A, G, VA, N, 0.1, 0.9, 7, 1, peer, 4.0)
    O.round_(Bm, G, VB, N, 0.1, 0.9, 7, 1, peer, 4.0, mix_first=True)
    m = np.zeros(N, bool); m[idx[:K]] = True
    assert np.array_equal(VA, VB)                                                   # the buffer never sees the exchange
    assert np.array_equal(A[:, ~m], Bm[:, ~m]) and np.array_equal(A[2:], Bm[2:])
    assert not np.array_equal(A[:2, m], Bm[:2, m])
    # under Eq. (7) the pair keeps a difference of gamma * (v_p - v_i) on masked coordinates; under Alg. 2 none
    assert np.array_equal(A[0, m], A[1, m]) and not np.array_equal(Bm[0, m], Bm[1, m])
    # without gradients both orders are the same exchange
    C1, C2 = X.copy(), X.copy()
    O.round_(C1, None, None, N, 0, 0, 7, 1, peer, 4.0); O.round_(C2, None, None, N, 0, 0, 7, 1, peer, 4.0, mix_first=True)
    assert np.array_equal(C1, C2)


# ------------------------------------------------- several local steps between exchanges
@pytest.mark.parametrize("mix_first", [False, True], ids=["alg2_order", "recursion_order"])
def test_tau_local_steps_then_one_exchange_equals_explicit_matrix_form(mix_first):
    # Communication period tau = 3: two rounds with W = I (a worker that only runs procedure SGD of Alg. 2)
    # and one round with the matching's W.  Composition used by callers: (tau - 1) x sgd_step, then round.
    n, N, c, tau = 4, 64, 2, 3
    rng = np.random.default_rng(55)
    lr = np.float32(0.125)
    for rnd, peer in enumerate(_matchings4(), start=1):
        X = rng.standard_normal((n, N)).astype(np.float32)
        Gs = [rng.standard_normal((n, N)).astype(np.float32) for _ in range(tau)]
        m = _mask_indep(N, 6, rnd, c)
        M = np.repeat(m[:, None], n, axis=1).astype(np.float64)
        W = _W(peer)
        step = lambda A, G: (A.astype(np.float64) - np.float64(lr) * G.astype(np.float64)).astype(np.float32)
        mix = lambda A: (A.T.astype(np.float64) * (1 - M) + (A.T.astype(np.float64) * M) @ W).T.astype(np.float32)
        want = X
        for G in Gs[:-1]:
            want = step(want, G)                                  # X o notM + (X o M) I - gamma G = X - gamma G
        sent = want if mix_first else step(want, Gs[-1])
        want = step(mix(want), Gs[-1]) if mix_first else mix(step(want, Gs[-1]))
        got = X.copy()
        for G in Gs[:-1]:
            assert O.sgd_step(got, G, None, float(lr), 0.0) == O.OK
        rc, K, idx, msg = O.round_(got, Gs[-1], None, N, float(lr), 0.0, 6, rnd, np.array(peer), float(c), mix_first=mix_first)
        assert rc == O.OK and K == int(m.sum())
        assert np.array_equal(msg[:, :K], sent[:, m])
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        # the same thing said with rounds only: an identity matching is a round without exchange
        alt = X.copy()
        for G in Gs[:-1]:
            O.round_(alt, G, None, N, float(lr), 0.0, 6, 1000 + rnd, np.arange(n), float(c), mix_first=mix_first)
        O.round_(alt, Gs[-1], None, N, float(lr), 0.0, 6, rnd, np.array(peer), float(c), mix_first=mix_first)
        assert np.array_equal(alt.view(np.uint32), want.view(np.uint32))
