"""Pins of the oracle's per-segment paths (one compression ratio per segment of the flat model) — CPU only.

The paper has one ratio c for the whole model (Sec. II-B); the segment table is this build's
extension.  Every expected value below comes from the second, pure-Python statement of the mask
rule (independent_philox) and from the explicit matrices of Eq. (2), Eq. (3) and the recursion of
Sec. III (Eq. (7)) with a mask matrix M whose rows follow the segment table; the oracle is never
asked to confirm itself.
"""
import numpy as np
import pytest

import independent_philox as IP
from oracle import saps_oracle as O

# cuts that are not multiples of 4, an empty segment, one- and two-element segments, c = 1 next to c = 1000,
# and equal ratios in neighbouring segments
LAYOUTS = [
    ([0, 3, 10, 10, 11, 13, 61, 64], [1000.0, 1.0, 7.0, 2.0, 1.0, 4.0, 2.0]),
    ([0, 1, 2, 40, 61], [1.0, 1000.0, 2.0, 2.0]),
    ([0, 0, 5, 5, 64], [2.0, 1.0, 3.0, 4.0]),
    ([0, 17, 50], [4.0, 1.0]),
]


def _mask_indep_seg(N, seed, rnd, off, cs):
    m = np.zeros(N, dtype=bool)
    for s, c in enumerate(cs):
        T = int(2**32 / c)
        for j in range(off[s], off[s + 1]):
            m[j] = IP.coord_bits(seed, rnd, j) < T
    return m


def _W(peer):
    n = len(peer)
    W = np.zeros((n, n))
    for i, p in enumerate(peer):
        if p == i:
            W[i, i] = 1.0
        else:
            W[i, i] = W[i, p] = 0.5
    return W


PEERS4 = [[1, 0, 3, 2], [2, 3, 0, 1], [3, 2, 1, 0], [1, 0, 2, 3], [0, 1, 2, 3]]


@pytest.mark.parametrize("off,cs", LAYOUTS, ids=[f"layout{i}" for i in range(len(LAYOUTS))])
def test_mask_compact_with_segments_matches_the_independent_mask(off, cs):
    N, n = off[-1], 3
    rng = np.random.default_rng(N)
    X = rng.standard_normal((n, N + 3)).astype(np.float32)            # ld > N: padding never packed
    for seed, rnd in [(0, 1), (7, 2), (2**40 + 1, 2**33 + 5)]:
        m = _mask_indep_seg(N, seed, rnd, off, cs)
        rc, K, idx, msg = O.mask_compact(X, N, seed, rnd, cs, off)
        assert rc == O.OK
        assert K == int(m.sum())
        assert np.array_equal(idx[:K], np.flatnonzero(m).astype(np.uint32))
        assert np.array_equal(msg[:, :K].view(np.uint32), X[:, :N][:, m].view(np.uint32))
        assert not idx[K:].any() and not msg[:, K:].any()
        # segments with c = 1 are kept whole
        for s, c in enumerate(cs):
            if c == 1.0:
                assert m[off[s]:off[s + 1]].all()


def test_mask_compact_with_segments_at_model_scale():
    # several tiles' worth of coordinates; a 10-element segment like a classifier bias between two big ones
    N = 30_011
    off = [0, 3, 10, 10, 4099, 4109, 20_001, N]
    cs = [1.0, 2.0, 7.0, 100.0, 1.0, 10.0, 1000.0]
    X = np.random.default_rng(1).standard_normal((2, N)).astype(np.float32)
    m = _mask_indep_seg(N, 9, 2, off, cs)
    rc, K, idx, msg = O.mask_compact(X, N, 9, 2, cs, off)
    assert rc == O.OK and K == int(m.sum())
    assert np.array_equal(idx[:K], np.flatnonzero(m).astype(np.uint32))
    assert np.array_equal(msg[:, :K], X[:, m])
    for s in range(len(cs)):
        L = off[s + 1] - off[s]
        p = 1 / cs[s]
        inside = int(((idx[:K] >= off[s]) & (idx[:K] < off[s + 1])).sum())
        if L > 500:
            assert abs(inside - L * p) <= 5 * np.sqrt(L * p * (1 - p))
        if cs[s] == 1.0:
            assert inside == L


@pytest.mark.parametrize("mix_first", [False, True], ids=["alg2_order", "recursion_order"])
@pytest.mark.parametrize("off,cs", LAYOUTS, ids=[f"layout{i}" for i in range(len(LAYOUTS))])
def test_round_with_segments_equals_explicit_matrix_form(off, cs, mix_first):
    # Exchange only and with a plain local step, against X o notM + (X o M) W [- gamma G] where the
    # rows of M follow the segment table (identical columns, Lemma 1's premise).
    N, n = off[-1], 4
    rng = np.random.default_rng(3 * N + int(mix_first))
    lr = np.float32(0.25)
    for rnd, peer in enumerate(PEERS4, start=1):
        X = rng.standard_normal((n, N)).astype(np.float32)
        G = rng.standard_normal((n, N)).astype(np.float32)
        m = _mask_indep_seg(N, 11, rnd, off, cs)
        M = np.repeat(m[:, None], n, axis=1).astype(np.float64)        # N x n, columns = workers
        W = _W(peer)

        def mix(A32):
            Ap = A32.T.astype(np.float64)
            return (Ap * (1 - M) + (Ap * M) @ W).T.astype(np.float32)

        # exchange only
        got = X.copy()
        rc, K, idx, msg = O.round_(got, None, None, N, 0.0, 0.0, 11, rnd, np.array(peer), cs, off, mix_first=mix_first)
        assert rc == O.OK and K == int(m.sum())
        assert np.array_equal(idx[:K], np.flatnonzero(m).astype(np.uint32))
        assert np.array_equal(msg[:, :K], X[:, m])
        assert np.array_equal(got.view(np.uint32), mix(X).view(np.uint32))
        # with the local step (plain SGD: one rounding per coordinate, exact in float64 before it)
        step = lambda A32: (A32.astype(np.float64) - np.float64(lr) * G.astype(np.float64)).astype(np.float32)
        want = step(mix(X)) if mix_first else mix(step(X))
        sent = X if mix_first else step(X)
        got = X.copy()
        rc, K, idx, msg = O.round_(got, G, None, N, float(lr), 0.0, 11, rnd, np.array(peer), cs, off, mix_first=mix_first)
        assert rc == O.OK and K == int(m.sum())
        assert np.array_equal(idx[:K], np.flatnonzero(m).astype(np.uint32))
        assert np.array_equal(msg[:, :K], sent[:, m])
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("mix_first", [False, True], ids=["alg2_order", "recursion_order"])
def test_capacity_rule_counts_with_each_segments_own_ratio(mix_first):
    # first segment nearly empty (c = 1000), second kept whole (c = 1): K = about 2 + 300.  A count that
    # used the first ratio everywhere would see K of about 0 and go on to write.
    N = 2300
    off, cs = [0, 2000, N], [1000.0, 1.0]
    m = _mask_indep_seg(N, 4, 1, off, cs)
    K_true = int(m.sum())
    assert K_true >= 300
    X0 = np.random.default_rng(5).standard_normal((2, N)).astype(np.float32)
    G = np.ones_like(X0); V0 = np.zeros_like(X0)
    for cap, want_rc in [(K_true - 1, O.ECAPACITY), (K_true, O.OK)]:
        X, V = X0.copy(), V0.copy()
        rc, K, idx, msg = O.round_(X, G, V, N, 0.1, 0.9, 4, 1, np.array([1, 0]), cs, off, msg_ld=cap, mix_first=mix_first)
        assert rc == want_rc and K == K_true
        if want_rc == O.ECAPACITY:
            assert np.array_equal(X, X0) and not V.any() and not idx.any() and not msg.any()
        else:
            assert np.array_equal(idx[:K], np.flatnonzero(m).astype(np.uint32))
    # and the reverse: first segment kept whole, the rest nearly empty
    cs2 = [1.0, 1000.0]
    m2 = _mask_indep_seg(N, 4, 1, off, cs2)
    X = X0.copy()
    rc, K, idx, msg = O.round_(X, None, None, N, 0, 0, 4, 1, np.array([1, 0]), cs2, off, msg_ld=int(m2.sum()), mix_first=mix_first)
    assert rc == O.OK and K == int(m2.sum()) and K < N
    assert np.array_equal(idx[:K], np.flatnonzero(m2).astype(np.uint32))


def test_uniform_table_equals_scalar_ratio():
    # a table whose segments all carry the same ratio is the paper's single-c mask
    N = 5000
    a = O.mask(N, 3, 8, 10.0)
    b = O.mask(N, 3, 8, [10.0] * 4, [0, 7, 1001, 1002, N])
    ref = np.array([IP.keep(3, 8, j, 10) for j in range(N)], dtype=np.uint8)
    assert np.array_equal(a, ref) and np.array_equal(b, ref)
