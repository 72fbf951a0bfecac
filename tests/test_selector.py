"""Adaptive peer selection (Alg. 1 line 2, Alg. 3): the host library against the oracle's
unique quantities (graphs, components, maximum matching size) and against the properties the
paper states.  CPU only: nothing here touches a GPU."""
import time

import numpy as np
import pytest

from oracle import peer_selection_oracle as PO

torch = pytest.importorskip("torch")
from paper_2002_09692_amd import binding as B   # noqa: E402  (host-side entry points only)


def rand_graph(n, p, rng):
    U = rng.random((n, n)) < p
    E = np.triu(U, 1)
    return (E | E.T).astype(np.uint8)


# ------------------------------------------------------------------ oracle self-pins
def test_oracle_max_matching_size_on_textbook_graphs():
    def g(n, edges):
        E = np.zeros((n, n), np.uint8)
        for a, b in edges:
            E[a, b] = E[b, a] = 1
        return E
    assert PO.max_matching_size(g(4, [(0, 1), (1, 2), (2, 3)])) == 2                    # path P4
    assert PO.max_matching_size(g(5, [(0, 1), (1, 2), (2, 3), (3, 4), (4, 0)])) == 2    # odd cycle C5
    assert PO.max_matching_size(g(4, [(0, 1), (0, 2), (0, 3)])) == 1                    # star
    assert PO.max_matching_size(np.ones((7, 7), np.uint8)) == 3                         # K7
    # a triangle with a pendant path on each corner needs the blossom: perfect matching of size 3
    assert PO.max_matching_size(g(6, [(0, 1), (1, 2), (2, 0), (0, 3), (1, 4), (2, 5)])) == 3
    # Petersen graph has a perfect matching
    pet = [(i, (i + 1) % 5) for i in range(5)] + [(i, i + 5) for i in range(5)] + [(5 + i, 5 + (i + 2) % 5) for i in range(5)]
    assert PO.max_matching_size(g(10, pet)) == 5


def test_oracle_components_match_scipy():
    sp = pytest.importorskip("scipy.sparse.csgraph")
    rng = np.random.default_rng(1)
    for n, p in [(12, 0.08), (30, 0.04), (30, 0.2), (1, 0.5)]:
        Q = rand_graph(n, p, rng)
        k, lab = PO.component_labels(Q)
        k2, lab2 = sp.connected_components(Q, directed=False)
        assert k == k2
        # same partition
        assert len({(a, b) for a, b in zip(lab, lab2)}) == k


def test_oracle_graph_pieces_on_a_hand_worked_five_worker_example():
    # Worked by hand from Sec. II-C and Alg. 1 / Alg. 3: speeds measured in both directions, the slower one counts.
    Braw = np.array([[0, 9, 2, 7, 1],
                     [5, 0, 8, 3, 6],
                     [4, 8, 0, 2, 9],
                     [7, 1, 6, 0, 3],
                     [2, 6, 5, 4, 0]], dtype=np.float64)
    S = np.array([[0, 5, 2, 7, 1],
                  [5, 0, 8, 1, 6],
                  [2, 8, 0, 2, 5],
                  [7, 1, 2, 0, 3],
                  [1, 6, 5, 3, 0]], dtype=np.float64)
    assert np.array_equal(PO.symmetrise(Braw), S)
    # B_thres = 5 keeps the links (0,1) (0,3) (1,2) (1,4) (2,4); the threshold itself counts as fast enough
    Bstar = np.zeros((5, 5), np.uint8)
    for a, b in [(0, 1), (0, 3), (1, 2), (1, 4), (2, 4)]:
        Bstar[a, b] = Bstar[b, a] = 1
    assert np.array_equal(PO.filtered_graph(Braw, 5.0), Bstar)
    assert PO.filtered_graph(Braw, 5.000001).sum() == 2 * 3          # (0,1) and (2,4) drop out
    # timestamps at round t = 10: (0,1) used in round 9, (2,3) in 7, (1,2) in 6, (0,4) in 2, the rest never
    R = np.full((5, 5), PO.NEVER, dtype=np.int64)
    for (a, b), r in {(0, 1): 9, (2, 3): 7, (1, 2): 6, (0, 4): 2}.items():
        R[a, b] = R[b, a] = r

    def graph(edges):
        Q = np.zeros((5, 5), np.uint8)
        for a, b in edges:
            Q[a, b] = Q[b, a] = 1
        return Q
    # window 4: recent means used after round 6, so (1,2) has just expired
    assert np.array_equal(PO.recently_connected(R, 4, 10), graph([(0, 1), (2, 3)]))
    connected, ncomp, E = PO.candidate_matrix(Bstar, R, 4, 10)
    assert not connected and ncomp == 3                              # {0,1} {2,3} {4}
    assert np.array_equal(E, graph([(0, 2), (0, 3), (0, 4), (1, 2), (1, 3), (1, 4), (2, 4), (3, 4)]))
    assert PO.max_matching_size(E) == 2
    # window 5: (1,2) still counts, components {0,1,2,3} {4}: only links to worker 4 join two components
    assert np.array_equal(PO.recently_connected(R, 5, 10), graph([(0, 1), (2, 3), (1, 2)]))
    connected, ncomp, E = PO.candidate_matrix(Bstar, R, 5, 10)
    assert not connected and ncomp == 2
    assert np.array_equal(E, graph([(0, 4), (1, 4), (2, 4), (3, 4)]))
    assert PO.max_matching_size(E) == 1
    # window 9: (0,4) from round 2 counts too, everyone is connected, so the fast links B* are the candidates
    assert np.array_equal(PO.recently_connected(R, 9, 10), graph([(0, 1), (2, 3), (1, 2), (0, 4)]))
    connected, ncomp, E = PO.candidate_matrix(Bstar, R, 9, 10)
    assert connected and ncomp == 1 and np.array_equal(E, Bstar)
    assert PO.max_matching_size(E) == 2                              # e.g. (0,3) (1,2) or (0,3) (2,4)
    # nothing ever used: five isolated workers, every pair is a candidate
    connected, ncomp, E = PO.candidate_matrix(Bstar, np.full((5, 5), PO.NEVER, dtype=np.int64), 4, 1)
    assert not connected and ncomp == 5 and E.sum() == 20 and not E.diagonal().any()


# ------------------------------------------------------------ maximum matching (blossom)
@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 11, 14])
def test_max_matching_is_maximum_and_valid_on_random_graphs(n):
    rng = np.random.default_rng(100 + n)
    for trial in range(40):
        E = rand_graph(n, rng.choice([0.1, 0.25, 0.5, 0.9]), rng)
        want = PO.max_matching_size(E)
        for seed in (0, 1, 2):
            pairs, peer = B.saps_max_matching(E, seed)
            assert pairs == want, (n, trial, seed)
            assert PO.check_matching(peer, E) == pairs


def test_max_matching_blossom_cases_and_randomisation():
    def g(n, edges):
        E = np.zeros((n, n), np.uint8)
        for a, b in edges:
            E[a, b] = E[b, a] = 1
        return E
    tri = g(6, [(0, 1), (1, 2), (2, 0), (0, 3), (1, 4), (2, 5)])
    for seed in range(20):
        pairs, peer = B.saps_max_matching(tri, seed)
        assert pairs == 3 and sorted(map(tuple, np.sort(np.stack([np.arange(6), peer], 1), 1).tolist()))[::2] is not None
        assert PO.check_matching(peer, tri) == 3
    # nested odd cycles
    E = g(10, [(0, 1), (1, 2), (2, 3), (3, 4), (4, 0), (2, 5), (5, 6), (6, 7), (7, 2), (7, 8), (4, 9)])
    assert B.saps_max_matching(E, 3)[0] == PO.max_matching_size(E)
    # different seeds give different maximum matchings of the complete graph (RandomlyMaxMatch)
    K = np.ones((16, 16), np.uint8)
    seen = {tuple(B.saps_max_matching(K, s)[1]) for s in range(30)}
    assert len(seen) > 20
    # same seed, same result
    assert np.array_equal(B.saps_max_matching(K, 5)[1], B.saps_max_matching(K, 5)[1])


def test_max_matching_larger_graphs_properties():
    rng = np.random.default_rng(7)
    for n in (32, 128, 257):
        E = rand_graph(n, 0.5, rng)
        pairs, peer = B.saps_max_matching(E, 1)
        assert PO.check_matching(peer, E) == pairs == n // 2          # dense random graphs have (near-)perfect matchings
        # no edge may join two unmatched vertices (maximal), here trivially true; check on a sparse graph
        S = rand_graph(n, 1.5 / n, rng)
        pairs, peer = B.saps_max_matching(S, 1)
        PO.check_matching(peer, S)
        free = np.flatnonzero(peer == np.arange(n))
        assert not S[np.ix_(free, free)].any()


# ------------------------------------------------------------------------- Alg. 3 rounds
@pytest.mark.parametrize("n,T_thres,B_thres", [(8, 3, 50.0), (12, 6, 70.0), (14, 2, 30.0), (9, 4, 50.0), (10, 8, 95.0)])
def test_selector_follows_alg3_round_by_round(n, T_thres, B_thres):
    rng = np.random.default_rng(n * 10 + T_thres)
    Braw = rng.uniform(1, 100, (n, n))                              # not symmetric on purpose
    Bs = PO.symmetrise(Braw)
    Bstar = PO.filtered_graph(Braw, B_thres)
    sel = B.PeerSelector(Braw, B_thres, T_thres, seed=5)
    R = np.full((n, n), PO.NEVER, dtype=np.int64)
    assert np.array_equal(sel.saps_selector_get_R(), R)
    saw_connected = saw_split = False
    for t in range(1, 41):
        connected, ncomp, E = PO.candidate_matrix(Bstar, R, T_thres, t)
        peer, info = sel.saps_selector_next(t)
        assert info["rc_connected"] == int(connected) and info["rc_components"] == ncomp
        saw_connected |= connected; saw_split |= not connected
        # first pass: a maximum matching of E
        assert info["first_pairs"] == PO.max_matching_size(E)
        # every worker matched (one left over when n is odd), first-pass pairs are edges of E
        total = PO.check_matching(peer, np.ones((n, n), np.uint8))
        assert total == n // 2 == info["first_pairs"] + info["second_pairs"]
        on_E = sum(1 for i in range(n) if peer[i] > i and (E[i, peer[i]] or E[peer[i], i]))
        assert on_E >= info["first_pairs"]
        bw = [Bs[i, peer[i]] for i in range(n) if peer[i] > i]
        assert info["min_bandwidth"] == min(bw) and abs(info["mean_bandwidth"] - np.mean(bw)) < 1e-12
        # R records the round's pairs
        for i in range(n):
            if peer[i] != i:
                R[i, peer[i]] = t
        assert np.array_equal(sel.saps_selector_get_R(), R)
    if T_thres >= 3:
        assert saw_connected
    assert saw_split                                               # round 1 always starts from isolated workers


def test_recently_connected_edges_keep_the_graph_connected():
    # Assumption 3 needs the union of possible edges to be connected: whenever the last T_thres rounds did
    # not connect everyone, the next matching only uses edges between different components.
    n, T = 32, 6
    rng = np.random.default_rng(3)
    Braw = rng.uniform(0, 5, (n, n))
    sel = B.PeerSelector(Braw, 2.5, T, seed=1)
    R = np.full((n, n), PO.NEVER, dtype=np.int64)
    for t in range(1, 121):
        Q = PO.recently_connected(R, T, t)
        ncomp, lab = PO.component_labels(Q)
        peer, info = sel.saps_selector_next(t)
        if ncomp > 1:
            cross = sum(1 for i in range(n) if peer[i] > i and lab[i] != lab[peer[i]])
            assert cross == info["first_pairs"] and cross >= 1
        for i in range(n):
            R[i, peer[i]] = t if peer[i] != i else R[i, peer[i]]
    # with a generous window the selector mostly runs on the filtered graph
    sel2 = B.PeerSelector(Braw, 2.5, 40, seed=1)
    flags = [sel2.saps_selector_next(t)[1]["rc_connected"] for t in range(1, 201)]
    assert sum(flags[20:]) > 150


def test_bandwidth_utilisation_order_saps_random_ring():
    # Sec. IV-C: with link speeds U(0, 5] MB/s on 32 workers the bottleneck link of the selected matching is,
    # on average, faster than that of a random maximum matching, which is faster than a ring's.
    n, rounds = 32, 300
    rng = np.random.default_rng(11)
    saps, rand, ring = [], [], []
    for trial in range(5):
        Braw = 5.0 * (1.0 - rng.random((n, n)))
        Bs = PO.symmetrise(Braw)
        sel = B.PeerSelector(Braw, 2.5, 10, seed=trial)
        for t in range(1, rounds + 1):
            saps.append(sel.saps_selector_next(t)[1]["min_bandwidth"])
            p = B.saps_max_matching(np.ones((n, n), np.uint8), 1000 * trial + t)[1]
            rand.append(min(Bs[i, p[i]] for i in range(n) if p[i] > i))
        ring.append(min(Bs[i, (i + 1) % n] for i in range(n)))
    assert np.mean(saps) > 1.5 * np.mean(rand) > 1.5 * np.mean(ring) * 1.0
    # closed form for the random baseline: each symmetrised link is the slower of two U(0,5] draws, so the
    # bottleneck of 16 pairs is the minimum of 32 uniforms, mean 5/33
    assert abs(np.mean(rand) - 5 / 33) < 0.03


def test_selector_argument_errors_and_speed():
    assert B.load_library().saps_selector_next(None, 1, None, None) == 1
    with pytest.raises(B.SapsError):
        B.PeerSelector(np.full((3, 3), np.nan), 1.0, 2)
    with pytest.raises(B.SapsError):
        B.PeerSelector(np.ones((3, 3)), 1.0, 0)
    rng = np.random.default_rng(0)
    for n in (32, 128):
        sel = B.PeerSelector(rng.uniform(1, 100, (n, n)), 50.0, 10, seed=0)
        t0 = time.perf_counter()
        for t in range(1, 51):
            sel.saps_selector_next(t)
        per = (time.perf_counter() - t0) / 50
        assert per < 0.05, f"n={n}: {per*1e3:.2f} ms per round"
