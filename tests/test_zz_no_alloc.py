"""saps_round_static (the entry point that allocates nothing, on the library's fixed scratch) against
saps_round on a context of the same layout, through the C ABI: bit-identical X, V, idx, msg and K on
calls in a row that share the one scratch array, each smaller than or different from the one before."""
import numpy as np
import pytest

from paper_2002_09692_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_09692_amd import binding
    binding.load_library()
    return binding


def _models(n, N, ld, seed, scale):
    rng = np.random.default_rng(seed)
    A = np.full((n, ld), 321.0, np.float32)
    A[:, :N] = scale * rng.standard_normal((n, N), dtype=np.float32)
    return A


def _bits(t):
    return t.cpu().numpy().view(np.uint32)


# (n, N, c, fused, with_v, pass idx, singles): the first case is the largest (group scan launched, N > 2^20),
# every later one is smaller, so stale counts of the earlier call lie behind the range the later one uses
CASES = [
    (8, 1_300_003, 100.0, True, True, True, 0),
    (4, 100_000, 100.0, True, True, True, 0),        # smaller, direct bases (no scan launch)
    (6, 70_001, 1000.0, False, False, False, 2),     # exchange only through the internal index list
    (5, 33_333, 8.0, False, False, True, 1),         # exchange only, tile walk; odd n
    (2, 2_001, 1.0, True, False, True, 0),           # c = 1: everything exchanged, plain SGD
]


def test_static_round_matches_context_round_on_calls_in_a_row(B):
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for rep in range(2):                                   # the whole sequence twice: big after small as well
            for case, (n, N, c, fused, with_v, give_idx, singles) in enumerate(CASES):
                ld = (N + 63) // 64 * 64
                cap = (int(N / c + 8 * np.sqrt(N / c) + 64) + 3) // 4 * 4 if c > 1 else (N + 3) // 4 * 4
                rng = np.random.default_rng(100 * rep + case)
                peer = synth.random_perfect_matching(n, rng)
                for i in rng.permutation(n)[:singles]:
                    p = peer[i]; peer[i], peer[p] = i, p
                seed, rnd = 77 + case, 5 + rep
                X0 = _models(n, N, ld, case, 0.05)
                G0 = _models(n, N, ld, case + 10, 1e-3) if fused else None
                V0 = _models(n, N, ld, case + 20, 1e-3) if with_v else None
                mu = 0.9 if with_v else 0.0
                out = []
                for which in ("context", "static"):
                    X = torch.from_numpy(X0).cuda()
                    G = None if G0 is None else torch.from_numpy(G0).cuda()
                    V = None if V0 is None else torch.from_numpy(V0).cuda()
                    idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda") if give_idx else None
                    msg = torch.full((n, cap), -5.0, dtype=torch.float32, device="cuda")
                    Kd = torch.full((1,), -1, dtype=torch.int64, device="cuda")
                    if which == "context":
                        with B.SapsContext(n, N, ld, cap, c, stream=stream) as ctx:
                            ctx.saps_round(X, G, V, 0.1, mu, seed, rnd, peer, idx, msg, Kd)
                            st, K = ctx.saps_poll_status()
                        assert st == 0 and 0 < K <= cap
                    else:
                        rc = B.saps_round_static(n, N, ld, c, cap, X, G, V, 0.1, mu, seed, rnd, peer, idx, msg, Kd, stream=stream)
                        assert rc == 0
                        stream.synchronize()
                    out.append((X, V, idx, msg, Kd))
                (Xc, Vc, ic, mc, Kc), (Xs, Vs, is_, ms, Ks) = out
                K = int(Kc.item())
                tag = f"rep {rep} case {case}"
                assert int(Ks.item()) == K, tag
                assert np.array_equal(_bits(Xs), _bits(Xc)), tag + " X"
                assert not np.array_equal(_bits(Xc), X0.view(np.uint32)), tag + " (the round did something)"
                if with_v:
                    assert np.array_equal(_bits(Vs), _bits(Vc)), tag + " V"
                if give_idx:
                    assert np.array_equal(_bits(is_), _bits(ic)), tag + " idx"
                assert np.array_equal(_bits(ms), _bits(mc)), tag + " msg"


def test_static_round_capacity_overflow_writes_nothing_and_reports_K(B):
    n, N, ld, c, cap = 2, 50_000, 50_048, 10.0, 1000            # K is about 5000 > cap
    X0 = _models(n, N, ld, 1, 0.05); G0 = _models(n, N, ld, 2, 1e-3)
    X = torch.from_numpy(X0).cuda(); G = torch.from_numpy(G0).cuda()
    idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    msg = torch.full((n, cap), -5.0, dtype=torch.float32, device="cuda")
    Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert B.saps_round_static(n, N, ld, c, cap, X, G, None, 0.1, 0.0, 3, 1, [1, 0], idx, msg, Kd) == 0
    torch.cuda.synchronize()
    assert int(Kd.item()) > cap
    assert np.array_equal(_bits(X), X0.view(np.uint32)) and bool((idx == -1).all()) and bool((msg == -5.0).all())
    # the next, fitting call is not disturbed by the skipped one
    cap2 = 6000
    idx2 = torch.full((cap2,), -1, dtype=torch.int32, device="cuda"); msg2 = torch.zeros((n, cap2), device="cuda")
    assert B.saps_round_static(n, N, ld, c, cap2, X, G, None, 0.1, 0.0, 3, 1, [1, 0], idx2, msg2, Kd) == 0
    Xr = torch.from_numpy(X0).cuda(); idx3 = torch.full((cap2,), -1, dtype=torch.int32, device="cuda"); msg3 = torch.zeros((n, cap2), device="cuda")
    K3 = torch.zeros(1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, cap2, c) as ctx:
        ctx.saps_round(Xr, G, None, 0.1, 0.0, 3, 1, [1, 0], idx3, msg3, K3)
        ctx.saps_poll_status()
    torch.cuda.synchronize()
    assert int(Kd.item()) == int(K3.item()) <= cap2
    assert np.array_equal(_bits(X), _bits(Xr)) and np.array_equal(_bits(idx2), _bits(idx3)) and np.array_equal(_bits(msg2), _bits(msg3))


def test_static_round_rejects_what_exceeds_its_limits(B):
    X = torch.zeros((2, 64), device="cuda"); Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    E = B.EINVAL
    big = (1 << 26) + 4
    # sizes beyond the scratch: refused on the host before anything touches X (its shape is not even looked at)
    L = B.load_library()
    import ctypes as C
    peer2 = np.array([1, 0], np.int32)
    def call(n, N, ld, c, msg_ld, peer, idx, Kp):
        return L.saps_round_static(n, N, ld, c, msg_ld, None, C.c_void_p(X.data_ptr()), None, None, 0.0, 0.0, 1, 1,
                                   peer.ctypes.data_as(C.c_void_p), idx, None, Kp)
    Kp = C.c_void_p(Kd.data_ptr())
    assert call(2, big, big, 100.0, 64, peer2, None, Kp) == E
    assert b"67,108,864" in L.saps_last_error(None)
    assert call(2, 64, 64, 0.5, 64, peer2, None, Kp) == E                         # c < 1
    assert call(2, 64, 64, 2.0, 64, peer2, None, None) == E                       # K_dev required
    assert call(2, 64, 64, 2.0, (1 << 19) + 4, peer2, None, Kp) == E              # internal list too small
    many = np.arange(300, dtype=np.int32)                                         # 300 unmatched workers = 300 units
    assert call(300, 64, 64, 2.0, 64, many, None, Kp) == E
    assert b"128 units" in L.saps_last_error(None)
    bad = np.array([1, 1], np.int32)
    assert call(2, 64, 64, 2.0, 64, bad, None, Kp) == B.EMATCH
    torch.cuda.synchronize()
    assert not X.any()
