"""End to end on the GPU: SAPS rounds (library kernels) around gradients of a synthetic decentralised
least-squares problem reach consensus at the joint optimum, and the whole trajectory is bit-identical to
the oracle's when both are fed the same gradients."""
import numpy as np
import pytest

from oracle import saps_oracle as O

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_09692_amd import binding
    binding.load_library()
    return binding


def test_decentralised_least_squares_converges_and_tracks_the_oracle(B):
    n, N, m, c, T = 8, 4096, 6144, 4.0, 300
    rng = np.random.default_rng(0)
    A = (rng.standard_normal((n, m, N)) / np.sqrt(m)).astype(np.float32)
    x_true = rng.standard_normal(N).astype(np.float32)
    b = (np.einsum("imj,j->im", A, x_true) + 0.01 * rng.standard_normal((n, m))).astype(np.float32)
    Ad, bd = torch.from_numpy(A).cuda(), torch.from_numpy(b).cuda()
    H = torch.einsum("imj,imk->jk", Ad.double(), Ad.double()) / n
    rhs = torch.einsum("imj,im->j", Ad.double(), bd.double()) / n
    x_star = torch.linalg.solve(H, rhs)
    X0 = rng.standard_normal((n, N)).astype(np.float32)
    X = torch.from_numpy(X0).cuda(); V = torch.zeros_like(X)
    Xo = X0.copy(); Vo = np.zeros_like(Xo)
    D = torch.zeros(2, dtype=torch.float64, device="cuda"); mean = torch.zeros(N, device="cuda")
    cap = 1200
    with B.SapsContext(n, N, N, cap, c) as ctx:
        ctx.saps_consensus(X, mean, D[0:1])
        err0 = float(torch.linalg.norm(mean.double() - x_star))
        for t in range(1, T + 1):
            perm = rng.permutation(n); peer = np.empty(n, np.int32)
            peer[perm[0::2]] = perm[1::2]; peer[perm[1::2]] = perm[0::2]
            r = torch.einsum("imj,ij->im", Ad, X) - bd               # each worker's residual at its own model
            G = torch.einsum("imj,im->ij", Ad, r).contiguous()       # its stochastic-gradient stand-in
            ctx.saps_round(X, G, V, 0.05, 0.9, 11, t, peer)
            if t <= 25:                                               # the oracle follows on the same gradients
                rc, *_ = O.round_(Xo, G.cpu().numpy(), Vo, N, 0.05, 0.9, 11, t, peer, c, msg_ld=cap * 2)
                assert rc == O.OK
                assert np.array_equal(X.cpu().numpy().view(np.uint32), Xo.view(np.uint32)), f"round {t}"
        ctx.saps_consensus(X, mean, D[1:2])
        assert ctx.saps_poll_status()[0] == 0
    d0, d1 = D.cpu().tolist()
    assert float(torch.linalg.norm(mean.double() - x_star)) < 0.02 * err0
    assert d1 < 1e-3 * d0
