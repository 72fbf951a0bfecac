"""GPU parity of round sequences in which the kernels of one round count the kept coordinates of the next
(saps.h, saps_round): whatever the order of (seed, round) pairs, whatever runs in between, and whether the
counts come from the previous call or from the call's own counting launch, every call must give the oracle's bits.
"""
import numpy as np
import pytest

from oracle import saps_oracle as O
from test_gpu_parity import assert_bits, dev, rand_models, rand_peer

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_09692_amd import binding
    binding.load_library()
    return binding


# (seed, round) in calling order: runs of consecutive rounds (the next round's counts are there), a repeated
# round, a jump, another seed with a round that would match, the wrap of the 64-bit round counter
SEQUENCE = [(7, 1), (7, 2), (7, 3), (7, 3), (7, 9), (7, 10), (8, 11), (8, 12), (7, 13), (7, 2**32 - 1), (7, 2**32),
            (7, 2**64 - 1), (7, 0), (7, 1)]


@pytest.mark.parametrize("kind", ["fused", "plain_sgd", "exchange_list", "exchange_walk", "exchange_hybrid", "mix_then_step"])
@pytest.mark.parametrize("shape", [(6, 70_001, 50.0), (4, 1_300_003, 1000.0), (5, 9_000, 3.0)])
def test_sequences_with_counts_prepared_by_the_previous_call(B, kind, shape):
    n, N, c = shape
    ld = (N + 63) // 64 * 64
    cap = min((int(N / c * 1.3) + 256) // 4 * 4, (N + 3) // 4 * 4)
    fused = kind in ("fused", "plain_sgd", "mix_then_step")
    mu = 0.9 if kind in ("fused", "mix_then_step") else 0.0
    X0 = rand_models(n, N, ld, 1)
    G0 = rand_models(n, N, ld, 2, scale=1e-3) if fused else None
    for prepare in (1, 0):
        Xo = X0.copy(); Vo = np.zeros_like(Xo) if mu else None
        X = dev(X0); G = dev(G0) if fused else None; V = torch.zeros_like(X) if mu else None
        idx = torch.zeros(cap, dtype=torch.int32, device="cuda"); msg = torch.zeros((n, cap), device="cuda")
        Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
        with B.SapsContext(n, N, ld, cap, c) as ctx:
            ctx.saps_set_tuning(B.TUNE_PREPARE_NEXT, prepare)
            path = {"exchange_list": 1, "exchange_walk": 2, "exchange_hybrid": 3}.get(kind)
            if path:
                ctx.saps_set_tuning(B.TUNE_EXCHANGE_PATH, path)
            for k, (seed, rnd) in enumerate(SEQUENCE):
                peer = rand_peer(n, 100 + k, singles=1 if n % 2 else 0)
                rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, 0.1, mu, seed, rnd, peer, c, msg_ld=cap,
                                               mix_first=(kind == "mix_then_step"))
                assert rc == O.OK
                if kind == "mix_then_step":
                    ctx.saps_round_ex(X, G, V, 0.1, mu, seed, rnd, peer, idx, msg, Kd, flags=B.ROUND_MIX_THEN_STEP)
                else:
                    ctx.saps_round(X, G, V, 0.1, mu, seed, rnd, peer, idx, msg, Kd)
                assert ctx.saps_poll_status() == (0, K), (k, seed, rnd)
                assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K]), (k, seed, rnd)
                assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], f"msg of call {k}")
                if k in (4, 8):
                    # calls of other entry points in between use and overwrite the count buffers
                    i2 = torch.zeros_like(idx); m2 = torch.zeros_like(msg)
                    ctx.saps_mask_compact(X, 99, 5, i2, m2, Kd)
                    assert ctx.saps_poll_status()[0] == 0
            assert_bits(X.cpu().numpy(), Xo, f"X (prepare={prepare})")
            if V is not None:
                assert_bits(V.cpu().numpy(), Vo, "V")


def test_capacity_overflow_in_a_prepared_sequence(B):
    """A round skipped for K > msg_ld still prepares the next one, and the next one is skipped or run on its own K."""
    n, N, ld, c = 4, 200_000, 200_000, 40.0
    Ks = [int(O.mask(N, 3, t, c).sum()) for t in range(1, 7)]
    cap = (sorted(Ks)[2] + 3) // 4 * 4                         # about half of the rounds fit
    X0 = rand_models(n, N, ld, 5)
    Xo = X0.copy(); X = dev(X0)
    Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    peer = rand_peer(n, 1)
    with B.SapsContext(n, N, ld, cap, c) as ctx:
        for t in range(1, 7):
            rc, K, _, _ = O.round_(Xo, None, None, N, 0.0, 0.0, 3, t, peer, c, msg_ld=cap)
            ctx.saps_round(X, None, None, 0.0, 0.0, 3, t, peer, None, None, Kd)
            st, Kg = ctx.saps_poll_status()
            assert Kg == Ks[t - 1] == int(Kd.item())
            assert (st == B.ECAPACITY) == (Ks[t - 1] > cap) == (rc == O.ECAPACITY)
            assert_bits(X.cpu().numpy(), Xo, f"X after round {t}")


def test_graph_replays_between_eager_rounds(B):
    """Calls recorded under stream capture count into their own buffers: replaying the graph between eager rounds
    neither disturbs what the eager rounds have prepared nor depends on it."""
    n, N, ld, c, cap = 6, 150_001, 150_016, 60.0, 3600
    X0h = rand_models(n, N, ld, 1); G0h = rand_models(n, N, ld, 2, scale=1e-3)
    peers = {t: rand_peer(n, 70 + t) for t in range(1, 12)}
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        X = dev(X0h); G = dev(G0h); V = torch.zeros_like(X)
        idx = torch.zeros(cap, dtype=torch.int32, device="cuda"); msg = torch.zeros((n, cap), device="cuda")
        Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    s.synchronize()
    Xo = X0h.copy(); Vo = np.zeros_like(Xo)

    def oracle(t):
        assert O.round_(Xo, G0h, Vo, N, 0.1, 0.9, 4, t, peers[t], c, msg_ld=cap)[0] == O.OK

    with B.SapsContext(n, N, ld, cap, c, stream=s) as ctx:
        def eager(t):
            ctx.saps_round(X, G, V, 0.1, 0.9, 4, t, peers[t], idx, msg, Kd)
            oracle(t)
        g = torch.cuda.CUDAGraph()
        eager(1); eager(2)                                     # round 3 is now prepared
        s.synchronize()
        with torch.cuda.graph(g, stream=s):                    # records rounds 3, 4, 5 (nothing runs yet)
            for t in (3, 4, 5):
                ctx.saps_round(X, G, V, 0.1, 0.9, 4, t, peers[t], idx, msg, Kd)
        g.replay()
        for t in (3, 4, 5):
            oracle(t)
        torch.cuda.synchronize()
        assert_bits(X.cpu().numpy(), Xo, "X after the first replay")
        eager(6); eager(7)                                     # eager rounds: 7 uses what 6 prepared
        torch.cuda.synchronize()
        assert_bits(X.cpu().numpy(), Xo, "X after eager rounds 6, 7")
        g.replay()                                             # rounds 3, 4, 5 again, on the current state
        for t in (3, 4, 5):
            oracle(t)
        eager(8)                                               # prepared by round 7, before the replay
        torch.cuda.synchronize()
        assert ctx.saps_poll_status()[0] == 0
        assert_bits(X.cpu().numpy(), Xo, "X after replay and eager round 8")
        assert_bits(V.cpu().numpy(), Vo, "V")
