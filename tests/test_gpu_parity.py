"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bars: K, idx, msg and averaged values bit-exact; the momentum update bit-exact under the
two-FMA reading and in any case within 1e-6 relative.
"""
import numpy as np
import pytest

from oracle import saps_oracle as O
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


def dev(a):
    return torch.from_numpy(a).cuda()


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def assert_bits(got, want, what):
    g, w = bits(got), bits(want)
    if not np.array_equal(g, w):
        bad = np.argwhere(g != w)
        raise AssertionError(f"{what}: {len(bad)} of {g.size} words differ, first at {bad[0]}: "
                             f"{got[tuple(bad[0])]!r} vs {want[tuple(bad[0])]!r}")


def rand_models(n, N, ld, seed, pad=777.0, scale=0.05):
    rng = np.random.default_rng(seed)
    X = np.full((n, ld), pad, np.float32)
    X[:, :N] = scale * rng.standard_normal((n, N), dtype=np.float32)
    return X


def rand_peer(n, seed, singles=0):
    rng = np.random.default_rng(seed)
    peer = synth.random_perfect_matching(n, rng)
    for i in rng.permutation(n)[:singles]:
        p = peer[i]
        peer[i], peer[p] = i, p
    return peer


def run_round_both(B, n, N, ld, seg_c, seg_off, seed, rnd, peer, fused, mu=0.9, lr=0.1, msg_ld=None, tuning=(),
                   with_v=True, outputs=True):
    X0 = rand_models(n, N, ld, 1)
    G0 = rand_models(n, N, ld, 2, pad=555.0, scale=1e-3) if fused else None
    V0 = rand_models(n, N, ld, 3, pad=333.0, scale=1e-3) if (fused and with_v) else None
    if msg_ld is None:
        msg_ld = (N + 3) // 4 * 4
    # oracle
    Xo = X0[:, :].copy(); Vo = None if V0 is None else V0.copy()
    rc_o, K_o, idx_o, msg_o = O.round_(Xo, G0, Vo, N, lr, mu if with_v else 0.0, seed, rnd, peer, seg_c, seg_off, msg_ld=msg_ld)
    # device
    X = dev(X0); G = None if G0 is None else dev(G0); V = None if V0 is None else dev(V0)
    idx = torch.full((max(msg_ld, 4),), -1, dtype=torch.int32, device="cuda") if outputs else None
    msg = torch.full((n, msg_ld), -5.0, dtype=torch.float32, device="cuda") if outputs else None
    Kd = torch.full((1,), -1, dtype=torch.int64, device="cuda") if outputs else None
    with B.SapsContext(n, N, ld, msg_ld, seg_c, seg_off) as ctx:
        for k, v in tuning:
            ctx.saps_set_tuning(k, v)
        ctx.saps_round(X, G, V, lr, mu if with_v else 0.0, seed, rnd, peer, idx, msg, Kd)
        st, K = ctx.saps_poll_status()
    return dict(rc_o=rc_o, K_o=K_o, idx_o=idx_o, msg_o=msg_o, Xo=Xo, Vo=Vo, st=st, K=K, X=X.cpu().numpy(),
                V=None if V is None else V.cpu().numpy(), idx=None if idx is None else idx.cpu().numpy().view(np.uint32),
                msg=None if msg is None else msg.cpu().numpy(), Kd=None if Kd is None else int(Kd.item()),
                X0=X0, V0=V0, msg_ld=msg_ld)


def check_round(r, N):
    assert r["rc_o"] == O.OK and r["st"] == 0
    K = r["K_o"]
    assert r["K"] == K
    if r["Kd"] is not None:
        assert r["Kd"] == K
        assert np.array_equal(r["idx"][:K], r["idx_o"][:K]), "idx"
        assert np.all(r["idx"][K:] == 0xFFFFFFFF), "idx written beyond K"
        assert_bits(r["msg"][:, :K], r["msg_o"][:, :K], "msg")
        assert np.all(r["msg"][:, K:] == -5.0), "msg written beyond K"
    assert_bits(r["X"], r["Xo"], "X")            # includes the padding columns: never touched
    if r["V"] is not None:
        assert_bits(r["V"], r["Vo"], "V")
        np.testing.assert_allclose(r["V"][:, :N], r["Vo"][:, :N], rtol=1e-6, atol=0)
    np.testing.assert_allclose(r["X"][:, :N], r["Xo"][:, :N], rtol=1e-6, atol=0)


# ------------------------------------------------------------------------------ stages
@pytest.mark.parametrize("N,ld", [(5000, 5056), (4096, 4096), (1023, 1024), (3, 4), (1, 4), (10_001, 10_004)])
@pytest.mark.parametrize("with_v", [True, False])
def test_sgd_step(B, N, ld, with_v):
    n = 3
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2, pad=9.0); V0 = rand_models(n, N, ld, 3, pad=8.0)
    Xo, Vo = X0.copy(), V0.copy()
    mu = 0.9 if with_v else 0.0
    assert O.sgd_step(Xo, G0, Vo if with_v else None, 0.1, mu, N=N) == O.OK
    X, G, V = dev(X0), dev(G0), dev(V0)
    with B.SapsContext(n, N, ld, 0) as ctx:
        ctx.saps_sgd_step(X, G, V if with_v else None, 0.1, mu)
        assert ctx.saps_poll_status()[0] == 0
    assert_bits(X.cpu().numpy(), Xo, "X")
    assert_bits(V.cpu().numpy(), Vo, "V")
    assert_bits(G.cpu().numpy(), G0, "G")


@pytest.mark.parametrize("N,c", [(100_000, 100.0), (5000, 4.0), (1030, 1.0), (2, 2.0), (50_001, 1000.0), (7777, 2.0**33)])
def test_mask_compact_then_merge(B, N, c):
    n = 5
    ld = (N + 63) // 64 * 64
    msg_ld = (N + 3) // 4 * 4
    X0 = rand_models(n, N, ld, 7)
    peer = rand_peer(n, 3)                                   # odd n: one worker unmatched
    rc, K, idx_o, msg_o = O.mask_compact(X0, N, 11, 4, c, msg_ld=msg_ld)
    assert rc == O.OK
    Xo = X0.copy()
    assert O.merge(Xo, N, peer, idx_o, msg_o, K) == O.OK
    X = dev(X0)
    idx = torch.full((max(msg_ld, 4),), -1, dtype=torch.int32, device="cuda")
    msg = torch.full((n, msg_ld), -5.0, device="cuda")
    Kd = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, msg_ld, c) as ctx:
        ctx.saps_mask_compact(X, 11, 4, idx, msg, Kd)
        assert ctx.saps_poll_status() == (0, K)
        assert_bits(X.cpu().numpy(), X0, "X after compaction (read only)")
        ctx.saps_merge(X, peer, idx, msg, Kd)
        assert ctx.saps_poll_status()[0] == 0
    assert int(Kd.item()) == K
    assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K])
    assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], "msg")
    assert np.all(msg.cpu().numpy()[:, K:] == -5.0)
    assert_bits(X.cpu().numpy(), Xo, "X after merge")


# ------------------------------------------------------------------------- whole round
SHAPES = [
    # n, N, ld, c
    (4, 100_000, 100_032, 100.0),      # several hundred tiles... ~98 tiles, N % 1024 != 0
    (6, 10_242, 10_304, 4.0),          # N % 4 == 2: ragged Philox block
    (5, 4097, 4100, 2.0),              # odd n, one coordinate into the 5th tile
    (2, 1024, 1024, 1.0),              # exactly one tile, everything exchanged
    (3, 5, 8, 1.0),                    # smaller than a tile and than a wave
    (2, 3, 4, 2.0),                    # smaller than one Philox block
    (8, 65_537, 65_600, 1000.0),       # very sparse
]


@pytest.mark.parametrize("n,N,ld,c", SHAPES)
@pytest.mark.parametrize("ppb", [1, 2, 8])
def test_fused_round_with_update(B, n, N, ld, c, ppb):
    peer = rand_peer(n, n + N, singles=1 if n > 2 else 0)
    r = run_round_both(B, n, N, ld, c, None, 5, 3, peer, fused=True, tuning=[(B.TUNE_PAIRS_PER_BLOCK, ppb)])
    check_round(r, N)


@pytest.mark.parametrize("knobs", [[(1, 1)], [(2, 0)], [(1, 1), (2, 0), (0, 4)]])
def test_fused_round_launch_knobs_do_not_change_results(B, knobs):
    n, N, ld = 6, 70_003, 70_016
    r = run_round_both(B, n, N, ld, 10.0, None, 8, 2, rand_peer(n, 1), fused=True, tuning=knobs)
    check_round(r, N)


def test_fused_round_without_momentum_buffer(B):
    n, N, ld = 4, 33_333, 33_344
    r = run_round_both(B, n, N, ld, 8.0, None, 1, 1, rand_peer(n, 2), fused=True, with_v=False)
    check_round(r, N)


def test_fused_round_without_optional_outputs(B):
    n, N, ld = 4, 20_000, 20_032
    r = run_round_both(B, n, N, ld, 16.0, None, 1, 9, rand_peer(n, 2), fused=True, outputs=False)
    check_round(r, N)


@pytest.mark.parametrize("n,N,ld,c", SHAPES)
@pytest.mark.parametrize("path", [1, 2, 3])
def test_exchange_only_round_both_paths(B, n, N, ld, c, path):
    peer = rand_peer(n, n * 3 + N, singles=1 if n > 2 else 0)
    r = run_round_both(B, n, N, ld, c, None, 2**40 + 17, 2**35 + 1, peer, fused=False, tuning=[(B.TUNE_EXCHANGE_PATH, path)])
    check_round(r, N)


@pytest.mark.parametrize("path", [1, 2, 3])
def test_exchange_only_without_optional_outputs(B, path):
    n, N, ld = 4, 30_000, 30_016
    r = run_round_both(B, n, N, ld, 50.0, None, 3, 3, rand_peer(n, 5), fused=False, outputs=False,
                       tuning=[(B.TUNE_EXCHANGE_PATH, path)])
    check_round(r, N)


@pytest.mark.parametrize("fused", [True, False])
def test_per_segment_ratios_at_unaligned_offsets(B, fused):
    n, N, ld = 4, 30_011, 30_016
    off = [0, 3, 10, 10, 4099, 20_001, N]
    cs = [1.0, 2.0, 7.0, 100.0, 10.0, 1000.0]
    r = run_round_both(B, n, N, ld, cs, off, 9, 2, rand_peer(n, 4), fused=fused)
    check_round(r, N)
    for path in (1, 2, 3):
        r = run_round_both(B, n, N, ld, cs, off, 9, 2, rand_peer(n, 4), fused=False, tuning=[(B.TUNE_EXCHANGE_PATH, path)])
        check_round(r, N)


def test_many_tiny_segments(B):
    # segments shorter than a tile, a wave and a Philox block (BN-sized tensors)
    rng = np.random.default_rng(0)
    sizes = rng.integers(1, 70, size=400).tolist() + [5000] + rng.integers(1, 9, size=300).tolist()
    off = synth.segment_offsets(sizes)
    N = int(off[-1]); ld = (N + 63) // 64 * 64
    cs = rng.choice([1.0, 3.0, 10.0, 100.0], size=len(sizes)).tolist()
    for fused in (True, False):
        r = run_round_both(B, 4, N, ld, cs, off, 4, 4, rand_peer(4, 9), fused=fused)
        check_round(r, N)


def test_identity_matching_and_all_singles(B):
    n, N, ld = 4, 9000, 9024
    r = run_round_both(B, n, N, ld, 4.0, None, 1, 1, np.arange(n, dtype=np.int32), fused=True)
    check_round(r, N)
    r = run_round_both(B, n, N, ld, 4.0, None, 1, 1, np.arange(n, dtype=np.int32), fused=False)
    check_round(r, N)
    assert_bits(r["X"], r["X0"], "identity matching without update changes nothing")


def test_fused_equals_unfused_sequence_on_device(B):
    n, N, ld, c = 6, 50_003, 50_048, 20.0
    msg_ld = 50_004
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2, scale=1e-3); V0 = rand_models(n, N, ld, 3, scale=1e-3)
    peer = rand_peer(n, 6)
    outs = []
    for fused in (True, False):
        X, G, V = dev(X0), dev(G0), dev(V0)
        idx = torch.zeros(msg_ld, dtype=torch.int32, device="cuda"); msg = torch.zeros((n, msg_ld), device="cuda")
        Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
        with B.SapsContext(n, N, ld, msg_ld, c) as ctx:
            if fused:
                ctx.saps_round(X, G, V, 0.1, 0.9, 4, 2, peer, idx, msg, Kd)
            else:
                ctx.saps_sgd_step(X, G, V, 0.1, 0.9)
                ctx.saps_mask_compact(X, 4, 2, idx, msg, Kd)
                ctx.saps_merge(X, peer, idx, msg, Kd)
            assert ctx.saps_poll_status()[0] == 0
        outs.append([t.cpu().numpy() for t in (X, V, idx, msg, Kd)])
    for a, b, name in zip(outs[0], outs[1], ["X", "V", "idx", "msg", "K"]):
        assert np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a, b.view(np.uint32) if b.dtype == np.float32 else b), name


def test_multi_round_trajectory_cfg1(B):
    # configuration 1: n=4, N=100000, c=100, 10 fused rounds, fresh gradients and a fresh matching per round
    wl = synth.workload("cfg1")
    ld = wl.ld(); cap = synth.recommended_capacity(wl)
    X0 = synth.make_models(wl, ld)
    Xo = X0.copy(); Vo = np.zeros_like(Xo)
    X = dev(X0); V = torch.zeros_like(X)
    idx = torch.zeros(cap, dtype=torch.int32, device="cuda"); msg = torch.zeros((wl.n, cap), device="cuda")
    Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    with B.SapsContext(wl.n, wl.N, ld, cap, 100.0) as ctx:
        for t in range(1, wl.rounds + 1):
            G0 = synth.make_grads(wl, t, ld); peer = wl.peers(t)
            rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, wl.N, wl.lr, wl.mu, 0, t, peer, 100.0, msg_ld=cap)
            assert rc == O.OK
            ctx.saps_round(X, dev(G0), V, wl.lr, wl.mu, 0, t, peer, idx, msg, Kd)
            assert ctx.saps_poll_status() == (0, K)
            assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K])
            assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], f"msg round {t}")
            assert_bits(X.cpu().numpy(), Xo, f"X round {t}")
            assert_bits(V.cpu().numpy(), Vo, f"V round {t}")


def test_c1_fixed_matching_pairs_become_identical(B):
    n, N, ld = 4, 5000, 5056
    X = dev(rand_models(n, N, ld, 1)); V = torch.zeros_like(X)
    peer = np.array([2, 3, 0, 1], np.int32)
    with B.SapsContext(n, N, ld, 5000, 1.0) as ctx:
        for t in range(1, 4):
            G = dev(rand_models(n, N, ld, 10 + t, scale=1e-3))
            ctx.saps_round(X, G, V, 0.1, 0.9, 1, t, peer)
            assert ctx.saps_poll_status() == (0, N)
            h = X.cpu().numpy()[:, :N]
            assert_bits(h[0], h[2], "pair (0,2)"); assert_bits(h[1], h[3], "pair (1,3)")
            assert not np.array_equal(h[0], h[1])


# --------------------------------------------------------------------- errors and edges
def test_capacity_overflow_skips_the_round(B):
    n, N, ld = 4, 40_000, 40_000
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2); V0 = rand_models(n, N, ld, 3)
    peer = rand_peer(n, 1)
    for fused in (True, False):
        for path in (1, 2, 3):
            X, G, V = dev(X0), dev(G0), dev(V0)
            idx = torch.full((100,), -1, dtype=torch.int32, device="cuda"); msg = torch.full((n, 100), -5.0, device="cuda")
            Kd = torch.full((1,), -1, dtype=torch.int64, device="cuda")
            with B.SapsContext(n, N, ld, 100, 2.0) as ctx:
                ctx.saps_set_tuning(B.TUNE_EXCHANGE_PATH, path)
                ctx.saps_round(X, G if fused else None, V if fused else None, 0.1, 0.9, 0, 1, peer, idx, msg, Kd)
                st, K = ctx.saps_poll_status()
                assert st == B.ECAPACITY and K == int(O.mask(N, 0, 1, 2.0).sum()) and int(Kd.item()) == K
                assert ctx.saps_poll_status()[0] == 0                      # flag is cleared by the poll
                # un-fused entries honour the same rule
                ctx.saps_mask_compact(X, 0, 1, idx, msg, Kd)
                ctx.saps_merge(X, peer, idx, msg, Kd)
                assert ctx.saps_poll_status()[0] == B.ECAPACITY
            assert_bits(X.cpu().numpy(), X0, "X"); assert_bits(V.cpu().numpy(), V0, "V")
            assert np.all(idx.cpu().numpy() == -1) and np.all(msg.cpu().numpy() == -5.0)


def test_host_side_argument_errors(B):
    n, N, ld = 4, 1000, 1000
    X = dev(rand_models(n, N, ld, 1))
    with pytest.raises(B.SapsError) as e:
        B.SapsContext(n, N, 999, 1000)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.SapsError):
        B.SapsContext(n, N, 1002, 1000)                        # ld % 4
    with pytest.raises(B.SapsError):
        B.SapsContext(n, N, ld, 1000, 0.5)                     # c < 1
    with pytest.raises(B.SapsError):
        B.SapsContext(n, N, ld, 1000, [2.0, 2.0], [0, 600, 999])   # segments do not end at N
    with pytest.raises(B.SapsError):
        B.SapsContext(n, N, ld, 1001)                          # capacity % 4
    with B.SapsContext(n, N, ld, 1000, 2.0) as ctx:
        for bad in ([1, 2, 0, 3], [0, 1, 2, 4], [-1, 1, 2, 3], [1, 1, 2, 3]):
            assert ctx.saps_round(X, None, None, 0, 0, 0, 1, np.array(bad), check=False) == B.EMATCH
            assert ctx.saps_merge(X, np.array(bad), torch.zeros(1000, dtype=torch.int32, device="cuda"),
                                  torch.zeros((n, 1000), device="cuda"), torch.zeros(1, dtype=torch.int64, device="cuda"),
                                  check=False) == B.EMATCH
        G = dev(rand_models(n, N, ld, 2))
        assert ctx.saps_round(X, G, None, 0.1, 0.9, 0, 1, np.array([1, 0, 3, 2]), check=False) == B.EINVAL
        assert ctx.saps_sgd_step(X, G, None, 0.1, 0.9, check=False) == B.EINVAL
        assert ctx.saps_set_tuning(0, 3, check=False) == B.EINVAL
        assert ctx.saps_set_tuning(99, 0, check=False) == B.EINVAL
        assert ctx.saps_poll_status()[0] == 0


def test_empty_model(B):
    n = 2
    X = torch.ones((n, 4), device="cuda")                     # N = 0 with a padded row stride of 4
    Kd = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, 0, 4, 0, 4.0) as ctx:
        ctx.saps_round(X, None, None, 0, 0, 1, 1, np.array([1, 0]), None, None, Kd)
        assert ctx.saps_poll_status() == (0, 0)
    assert int(Kd.item()) == 0 and bool((X == 1).all())


def test_special_values_travel_through_merge(B):
    n, N, ld = 2, 8, 8
    inf, nan, tiny = np.float32(np.inf), np.float32(np.nan), np.float32(1e-45)
    a = np.array([inf, inf, nan, -0.0, tiny, 3 * tiny, 3.4e38, 1.0], np.float32)
    b = np.array([1.0, -inf, 1.0, 0.0, tiny, tiny, 3.4e38, -1.0], np.float32)
    X0 = np.stack([a, b]); Xo = X0.copy()
    O.round_(Xo, None, None, N, 0, 0, 0, 1, np.array([1, 0]), 1.0)
    for path in (1, 2, 3):
        X = dev(X0)
        with B.SapsContext(n, N, ld, 8, 1.0) as ctx:
            ctx.saps_set_tuning(B.TUNE_EXCHANGE_PATH, path)
            ctx.saps_round(X, None, None, 0, 0, 0, 1, np.array([1, 0]))
            assert ctx.saps_poll_status() == (0, 8)
        h = X.cpu().numpy()
        assert np.array_equal(np.isnan(h), np.isnan(Xo))           # NaN payloads may differ between machines
        ok = ~np.isnan(Xo)
        assert np.array_equal(bits(h)[ok], bits(Xo)[ok])           # subnormals, signed zero, overflow to inf


@pytest.mark.parametrize("n", [257, 300])
def test_many_workers_unit_list_in_device_memory(B, n):
    # more than 128 units: the matching no longer fits the kernel arguments
    N, ld = 2051, 2112
    peer = rand_peer(n, 5, singles=3)
    for fused in (True, False):
        r = run_round_both(B, n, N, ld, 4.0, None, 6, 6, peer, fused=fused)
        check_round(r, N)
    # un-fused merge goes through the same list
    X0 = rand_models(n, N, ld, 1)
    rc, K, idx_o, msg_o = O.mask_compact(X0, N, 6, 6, 4.0, msg_ld=2052)
    Xo = X0.copy(); O.merge(Xo, N, peer, idx_o, msg_o, K)
    X = dev(X0); idx = torch.zeros(2052, dtype=torch.int32, device="cuda"); msg = torch.zeros((n, 2052), device="cuda")
    Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, 2052, 4.0) as ctx:
        for _ in range(6):                                     # more calls than staging slots
            X.copy_(torch.from_numpy(X0))
            ctx.saps_mask_compact(X, 6, 6, idx, msg, Kd)
            ctx.saps_merge(X, peer, idx, msg, Kd)
        assert ctx.saps_poll_status() == (0, K)
    assert_bits(X.cpu().numpy(), Xo, "X")


# ------------------------------------------------------------------ Eq. (7) ordering
@pytest.mark.parametrize("n,N,ld,c", SHAPES)
@pytest.mark.parametrize("with_v", [True, False])
def test_mix_then_step_round(B, n, N, ld, c, with_v):
    peer = rand_peer(n, n + 2 * N, singles=1 if n > 2 else 0)
    msg_ld = (N + 3) // 4 * 4
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2, pad=555.0, scale=1e-3)
    V0 = rand_models(n, N, ld, 3, pad=333.0, scale=1e-3) if with_v else None
    mu = 0.9 if with_v else 0.0
    Xo = X0.copy(); Vo = None if V0 is None else V0.copy()
    rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, 0.1, mu, 5, 3, peer, c, msg_ld=msg_ld, mix_first=True)
    assert rc == O.OK
    outs = []
    for fused in (True, False):
        X, G = dev(X0), dev(G0); V = None if V0 is None else dev(V0)
        idx = torch.full((max(msg_ld, 4),), -1, dtype=torch.int32, device="cuda")
        msg = torch.full((n, msg_ld), -5.0, device="cuda"); Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
        with B.SapsContext(n, N, ld, msg_ld, c) as ctx:
            if fused:
                ctx.saps_round_ex(X, G, V, 0.1, mu, 5, 3, peer, idx, msg, Kd, flags=B.ROUND_MIX_THEN_STEP)
            else:
                ctx.saps_mask_compact(X, 5, 3, idx, msg, Kd)
                ctx.saps_merge(X, peer, idx, msg, Kd)
                ctx.saps_sgd_step(X, G, V, 0.1, mu)
            assert ctx.saps_poll_status() == (0, K)
        assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K])
        assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], "msg")
        assert np.all(msg.cpu().numpy()[:, K:] == -5.0)
        assert_bits(X.cpu().numpy(), Xo, f"X fused={fused}")
        if with_v:
            assert_bits(V.cpu().numpy(), Vo, f"V fused={fused}")


@pytest.mark.parametrize("mix_first", [False, True], ids=["alg2_order", "recursion_order"])
@pytest.mark.parametrize("with_v", [True, False])
def test_tau_local_steps_between_exchanges(B, mix_first, with_v):
    # communication period tau = 3 over two periods: (tau - 1) x saps_sgd_step, then one saps_round(_ex)
    # with fresh gradients every step; the momentum buffer runs through local steps and rounds alike
    n, N, ld, c, tau, periods = 6, 70_003, 70_016, 20.0, 3, 2
    msg_ld = 4400
    X0 = rand_models(n, N, ld, 1); V0 = rand_models(n, N, ld, 3, pad=333.0, scale=1e-3) if with_v else None
    mu = 0.9 if with_v else 0.0
    Gs = [rand_models(n, N, ld, 50 + k, pad=555.0, scale=1e-3) for k in range(tau * periods)]
    peers = [rand_peer(n, 70 + r, singles=2 if r == 1 else 0) for r in range(periods)]
    Xo = X0.copy(); Vo = None if V0 is None else V0.copy()
    X = dev(X0); V = None if V0 is None else dev(V0)
    idx = torch.full((msg_ld,), -1, dtype=torch.int32, device="cuda")
    msg = torch.full((n, msg_ld), -5.0, device="cuda"); Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, msg_ld, c) as ctx:
        for r in range(periods):
            for k in range(tau - 1):
                G0 = Gs[r * tau + k]
                assert O.sgd_step(Xo, G0, Vo, 0.1, mu, N=N) == O.OK
                ctx.saps_sgd_step(X, dev(G0), V, 0.1, mu)
            G0 = Gs[r * tau + tau - 1]
            rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, 0.1, mu, 8, r + 1, peers[r], c, msg_ld=msg_ld, mix_first=mix_first)
            assert rc == O.OK
            ctx.saps_round_ex(X, dev(G0), V, 0.1, mu, 8, r + 1, peers[r], idx, msg, Kd,
                              flags=B.ROUND_MIX_THEN_STEP if mix_first else 0)
            assert ctx.saps_poll_status() == (0, K)
            assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K])
            assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], f"msg period {r}")
            assert_bits(X.cpu().numpy(), Xo, f"X period {r}")
            if with_v:
                assert_bits(V.cpu().numpy(), Vo, f"V period {r}")


def test_round_ex_rejects_unknown_flags_and_flag0_is_saps_round(B):
    n, N, ld = 4, 6000, 6016
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2, scale=1e-3); peer = rand_peer(n, 1)
    X = dev(X0); G = dev(G0); V = torch.zeros_like(X)
    with B.SapsContext(n, N, ld, 6000, 8.0) as ctx:
        assert ctx.saps_round_ex(X, G, V, 0.1, 0.9, 1, 1, peer, flags=2, check=False) == B.EINVAL
        ctx.saps_round_ex(X, G, V, 0.1, 0.9, 1, 1, peer, flags=0)
        X2 = dev(X0); V2 = torch.zeros_like(X2)
        ctx.saps_round(X2, G, V2, 0.1, 0.9, 1, 1, peer)
        assert ctx.saps_poll_status()[0] == 0
    assert torch.equal(X.view(torch.int32), X2.view(torch.int32)) and torch.equal(V.view(torch.int32), V2.view(torch.int32))


# ------------------------------------------------------------------- pipelined calls
@pytest.mark.parametrize("fused", [True, False])
def test_many_rounds_enqueued_without_host_synchronisation(B, fused):
    # 30 rounds back to back with no host synchronisation in between: the context's scratch is reused by
    # every call, so stream order alone must keep every round's K and the final state exact
    n, N, ld, c, rounds = 6, 150_003, 150_016, 20.0, 30
    cap = 9000
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2, scale=1e-3) if fused else None
    Xo = X0.copy(); Vo = np.zeros_like(Xo) if fused else None
    peers = [rand_peer(n, 100 + t, singles=t % 2) for t in range(rounds)]
    Ks_o = []
    for t in range(rounds):
        rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, 0.05, 0.9 if fused else 0.0, 77, t + 1, peers[t], c, msg_ld=cap)
        assert rc == O.OK
        Ks_o.append(K)
    X = dev(X0); G = dev(G0) if fused else None; V = torch.zeros_like(X) if fused else None
    idx = torch.zeros(cap, dtype=torch.int32, device="cuda"); msg = torch.zeros((n, cap), device="cuda")
    Ks = torch.full((rounds,), -1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, cap, c) as ctx:
        for t in range(rounds):
            ctx.saps_round(X, G, V, 0.05, 0.9 if fused else 0.0, 77, t + 1, peers[t], idx, msg, Ks[t:t + 1])
        assert ctx.saps_poll_status() == (0, Ks_o[-1])
    assert Ks.cpu().tolist() == Ks_o
    K = Ks_o[-1]
    assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K])
    assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], "msg")
    assert_bits(X.cpu().numpy(), Xo, "X")
    if fused:
        assert_bits(V.cpu().numpy(), Vo, "V")


def test_two_contexts_on_two_streams_do_not_disturb_each_other(B):
    n, N, ld, c = 4, 80_000, 80_000, 10.0
    cap = 9000
    X0 = rand_models(n, N, ld, 5); peer = rand_peer(n, 2)
    Xo = X0.copy()
    for t in range(1, 6):
        O.round_(Xo, None, None, N, 0, 0, 3, t, peer, c, msg_ld=cap)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    ctxs = []
    for s in (s1, s2):
        with torch.cuda.stream(s):
            X = dev(X0)
        s.synchronize()
        ctxs.append((B.SapsContext(n, N, ld, cap, c, stream=s), X))
    for t in range(1, 6):
        for ctx, X in ctxs:
            ctx.saps_round(X, None, None, 0, 0, 3, t, peer)
    for ctx, X in ctxs:
        assert ctx.saps_poll_status()[0] == 0
        assert_bits(X.cpu().numpy(), Xo, "X")
        ctx.close()


# --------------------------------------------------------------- seeded random sweep
def _random_case(rng):
    n = int(rng.integers(1, 12))
    N = int(rng.choice([rng.integers(1, 300), rng.integers(300, 6000), rng.integers(6000, 60_000)]))
    ld = (N + 3) // 4 * 4 + 4 * int(rng.integers(0, 20))
    nseg = int(rng.choice([1, 1, 2, 5, 40]))
    cuts = np.sort(rng.integers(0, N + 1, size=nseg - 1)) if nseg > 1 else np.array([], dtype=np.int64)
    off = np.concatenate([[0], cuts, [N]]).astype(np.int64)
    cs = rng.choice([1.0, 1.5, 2.0, 3.0, 10.0, 100.0, 1000.0, 1e9], size=nseg).tolist()
    peer = synth.random_perfect_matching(n, rng)
    for i in rng.permutation(n)[: int(rng.integers(0, 3))]:
        p = peer[i]; peer[i], peer[p] = i, p
    kind = str(rng.choice(["fused", "fused_nov", "mix_first", "exchange_list", "exchange_walk"]))
    return n, N, ld, off, cs, peer, kind, int(rng.integers(0, 2**63)), int(rng.integers(0, 2**63))


@pytest.mark.parametrize("case", range(60))
def test_random_configurations(B, case):
    rng = np.random.default_rng(5000 + case)
    n, N, ld, off, cs, peer, kind, seed, rnd = _random_case(rng)
    msg_ld = (N + 3) // 4 * 4
    X0 = rand_models(n, N, ld, case)
    fused = kind in ("fused", "fused_nov", "mix_first")
    G0 = rand_models(n, N, ld, case + 1, pad=1.5, scale=1e-2) if fused else None
    V0 = rand_models(n, N, ld, case + 2, pad=2.5, scale=1e-2) if kind in ("fused", "mix_first") else None
    mu = 0.9 if V0 is not None else 0.0
    Xo = X0.copy(); Vo = None if V0 is None else V0.copy()
    rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, 0.1, mu, seed, rnd, peer, cs, off, msg_ld=msg_ld, mix_first=(kind == "mix_first"))
    assert rc == O.OK
    X = dev(X0); G = None if G0 is None else dev(G0); V = None if V0 is None else dev(V0)
    idx = torch.full((max(msg_ld, 4),), -1, dtype=torch.int32, device="cuda")
    msg = torch.full((n, msg_ld), -5.0, device="cuda"); Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, msg_ld, cs, off) as ctx:
        if kind == "exchange_list":
            ctx.saps_set_tuning(B.TUNE_EXCHANGE_PATH, 1)
        if kind == "exchange_walk":
            ctx.saps_set_tuning(B.TUNE_EXCHANGE_PATH, 2)
            ctx.saps_set_tuning(B.TUNE_PAIRS_PER_BLOCK, int(rng.choice([1, 2, 4, 8])))
        if fused:
            ctx.saps_set_tuning(B.TUNE_PAIRS_PER_BLOCK, int(rng.choice([1, 2, 4, 8])))
        ctx.saps_round_ex(X, G, V, 0.1, mu, seed, rnd, peer, idx, msg, Kd, flags=B.ROUND_MIX_THEN_STEP if kind == "mix_first" else 0)
        assert ctx.saps_poll_status() == (0, K), (kind, n, N)
    assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K]), kind
    assert np.all(idx.cpu().numpy()[K:] == -1)
    assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], f"msg {kind}")
    assert np.all(msg.cpu().numpy()[:, K:] == -5.0)
    assert_bits(X.cpu().numpy(), Xo, f"X {kind} n={n} N={N} ld={ld}")
    if V is not None:
        assert_bits(V.cpu().numpy(), Vo, f"V {kind}")


def test_maximum_number_of_workers(B):
    # n = 65535 (the limit): 32767 pairs and one unmatched worker, unit list in device memory
    n, N, ld = 65535, 37, 40
    peer = rand_peer(n, 9)
    for fused in (True, False):
        r = run_round_both(B, n, N, ld, 2.0, None, 3, 3, peer, fused=fused)
        check_round(r, N)
    with pytest.raises(B.SapsError):
        B.SapsContext(65536, N, ld, 40, 2.0)


# ------------------------------------------------------------------ HIP graph capture
@pytest.mark.parametrize("fused", [True, False])
def test_round_loop_captured_in_a_graph_replays_like_eager(B, fused):
    # a round is only kernel launches when the matching fits the kernel arguments, so a loop of rounds can
    # be captured once and replayed; every replay must reproduce the eager result bit for bit
    n, N, ld, c, T = 8, 120_001, 120_064, 50.0, 6
    cap = 4000
    X0h = rand_models(n, N, ld, 1); G0h = rand_models(n, N, ld, 2, scale=1e-3)
    peers = [rand_peer(n, 40 + t) for t in range(T)]
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        X0 = dev(X0h); G = dev(G0h) if fused else None
        X = X0.clone(); V = torch.zeros_like(X) if fused else None
        idx = torch.zeros(cap, dtype=torch.int32, device="cuda"); msg = torch.zeros((n, cap), device="cuda")
        Ks = torch.zeros(T, dtype=torch.int64, device="cuda")
    s.synchronize()
    mu = 0.9 if fused else 0.0
    with B.SapsContext(n, N, ld, cap, c, stream=s) as ctx:
        def rounds():
            for t in range(T):
                ctx.saps_round(X, G, V, 0.1, mu, 9, t + 1, peers[t], idx, msg, Ks[t:t + 1])
        rounds()                                                   # eager
        assert ctx.saps_poll_status()[0] == 0
        ref = [a.clone() for a in (X, idx, msg, Ks)] + ([V.clone()] if fused else [])
        # against the oracle too
        Xo = X0h.copy(); Vo = np.zeros_like(Xo) if fused else None
        for t in range(T):
            O.round_(Xo, G0h if fused else None, Vo, N, 0.1, mu, 9, t + 1, peers[t], c, msg_ld=cap)
        assert_bits(X.cpu().numpy(), Xo, "eager X")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(s):
            X.copy_(X0)
            if fused:
                V.zero_()
        s.synchronize()
        with torch.cuda.graph(g, stream=s):
            rounds()
        for rep in range(4):
            with torch.cuda.stream(s):
                X.copy_(X0); idx.zero_(); msg.zero_(); Ks.zero_()    # eager work between the replays
                if fused:
                    V.zero_()
            s.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = [X, idx, msg, Ks] + ([V] if fused else [])
            for a, b in zip(got, ref):
                assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                                   b.view(torch.int32) if b.dtype == torch.float32 else b), f"replay {rep}"
        assert ctx.saps_poll_status()[0] == 0


def test_long_matching_is_refused_while_the_stream_is_capturing(B):
    # more than 128 units go through a pinned staging slot (an event wait and a copy), which a graph cannot
    # record faithfully: the call must say so instead of invalidating the capture or baking in a stale slot
    n, N, ld, cap = 300, 257, 320, 260
    peer = rand_peer(n, 3)                                        # 150 pairs > 128 units
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        X0 = dev(rand_models(n, N, ld, 1)); X = X0.clone()
        msg = torch.zeros((n, cap), device="cuda"); idx = torch.zeros(cap, dtype=torch.int32, device="cuda")
        Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    s.synchronize()
    with B.SapsContext(n, N, ld, cap, 2.0, stream=s) as ctx:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            X.add_(0.0)                                           # something to record
            rc_round = ctx.saps_round(X, None, None, 0.0, 0.0, 1, 1, peer, idx, msg, Kd, check=False)
            text = ctx._L.saps_last_error(ctx._h).decode()
            rc_merge = ctx.saps_merge(X, peer, idx, msg, Kd, check=False)
        assert rc_round == B.EINVAL and rc_merge == B.EINVAL and "capturing" in text
        g.replay(); torch.cuda.synchronize()
        assert torch.equal(X, X0)                                 # nothing of the round was recorded
        # outside a capture the same call works and matches the oracle
        ctx.saps_round(X, None, None, 0.0, 0.0, 1, 1, peer, idx, msg, Kd)
        assert ctx.saps_poll_status()[0] == 0
    Xo = X0.cpu().numpy().copy()
    rc, K, idx_o, msg_o = O.round_(Xo, None, None, N, 0.0, 0.0, 1, 1, peer, 2.0, msg_ld=cap)
    assert rc == O.OK and int(Kd.item()) == K
    assert_bits(X.cpu().numpy(), Xo, "X")


# ------------------------------------------------------------- optional outputs, lifetime
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("want", ["idx", "msg", "K"])
def test_each_optional_output_alone(B, fused, want):
    n, N, ld, c = 4, 45_001, 45_056, 30.0
    cap = 2000
    X0 = rand_models(n, N, ld, 3); G0 = rand_models(n, N, ld, 4, scale=1e-3) if fused else None
    peer = rand_peer(n, 8)
    Xo = X0.copy(); Vo = np.zeros_like(Xo) if fused else None
    rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, 0.1, 0.9 if fused else 0.0, 4, 4, peer, c, msg_ld=cap)
    X = dev(X0); G = dev(G0) if fused else None; V = torch.zeros_like(X) if fused else None
    idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda") if want == "idx" else None
    msg = torch.full((n, cap), -5.0, device="cuda") if want == "msg" else None
    Kd = torch.full((1,), -1, dtype=torch.int64, device="cuda") if want == "K" else None
    with B.SapsContext(n, N, ld, cap, c) as ctx:
        ctx.saps_round(X, G, V, 0.1, 0.9 if fused else 0.0, 4, 4, peer, idx, msg, Kd)
        assert ctx.saps_poll_status() == (0, K)
    assert_bits(X.cpu().numpy(), Xo, "X")
    if want == "idx":
        assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K]) and np.all(idx.cpu().numpy()[K:] == -1)
    if want == "msg":
        assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], "msg")
    if want == "K":
        assert int(Kd.item()) == K


def test_many_contexts_created_and_destroyed(B):
    X = dev(rand_models(2, 5000, 5056, 1))
    free0 = torch.cuda.mem_get_info()[0]
    for k in range(300):
        with B.SapsContext(2, 5000, 5056, 5000, 4.0) as ctx:
            if k % 50 == 0:
                ctx.saps_round(X, None, None, 0, 0, 1, k + 1, np.array([1, 0]))
                assert ctx.saps_poll_status()[0] == 0
    torch.cuda.synchronize()
    assert free0 - torch.cuda.mem_get_info()[0] < (64 << 20)          # contexts give their scratch back


# ------------------------------------------------------------------------------ list yardstick
@pytest.mark.parametrize("write_back", [False, True])
def test_list_probe_leaves_the_models_unchanged(B, write_back):
    n, N, ld = 6, 70_001, 70_016
    X0 = rand_models(n, N, ld, 11)
    cap = 2048
    X = dev(X0)
    idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    msg = torch.zeros((n, cap), dtype=torch.float32, device="cuda")
    Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, cap, 100.0) as ctx:
        ctx.saps_mask_compact(X, 3, 1, idx, msg, Kd)
        ctx.saps_list_probe(X, idx, Kd, write_back)
        # a foreign list with entries beyond N (and beyond ld) is skipped entry by entry
        bad = torch.tensor([0, 5, N, N + 1, ld + 100, 0x7FFFFFF0, N - 1] + [1] * (cap - 7), dtype=torch.int64).to(torch.int32).cuda()
        Kb = torch.tensor([7], dtype=torch.int64, device="cuda")
        ctx.saps_list_probe(X, bad, Kb, write_back)
        # K beyond the capacity: nothing happens
        Kbig = torch.tensor([cap + 1], dtype=torch.int64, device="cuda")
        ctx.saps_list_probe(X, idx, Kbig, write_back)
        st, _ = ctx.saps_poll_status()
    assert st == 0
    assert_bits(X.cpu().numpy(), X0, "X after the probe")


def test_list_exchange_store_policies_agree_with_the_oracle(B):
    """The list exchange picks write-back or streaming stores from the size of the lines a round touches:
    few rows take the first, many rows of a long model the second; both must give the oracle's bits."""
    for n, N, c in ((4, 300_000, 50.0), (64, 2_500_000, 20.0)):       # 4 x 8 k lines (4 MB), 64 x 63 k lines (0.52 GB)
        ld = (N + 63) // 64 * 64
        cap = int(N / c * 1.2) // 4 * 4
        r = run_round_both(B, n, N, ld, c, None, 9, 2, rand_peer(n, 5), fused=False, msg_ld=cap,
                           tuning=((B.TUNE_EXCHANGE_PATH, 1),))
        check_round(r, N)


@pytest.mark.parametrize("N", [1, 255, 4097, 70_001, 1_048_577, 1_300_000])
@pytest.mark.parametrize("c", [600.0, 1000.0, 20_000.0])
def test_index_list_of_sparse_masks(B, N, c):
    """Sparse masks take the index-list kernel in which one wave walks a whole group of 16 tiles: one group and
    less, ragged last groups, models below and above the size where the scan launch is skipped."""
    n = 2
    ld = (N + 63) // 64 * 64
    msg_ld = max(4, (int(N / c * 2) + 64) // 4 * 4)
    X0 = rand_models(n, N, ld, 7)
    for seed, rnd in ((1, 1), (2, 9)):
        rc, K, idx_o, msg_o = O.mask_compact(X0, N, seed, rnd, c, msg_ld=msg_ld)
        assert rc == O.OK
        X = dev(X0)
        idx = torch.full((msg_ld,), -1, dtype=torch.int32, device="cuda")
        msg = torch.full((n, msg_ld), -5.0, device="cuda")
        Kd = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        with B.SapsContext(n, N, ld, msg_ld, c) as ctx:
            ctx.saps_mask_compact(X, seed, rnd, idx, msg, Kd)
            assert ctx.saps_poll_status() == (0, K)
        assert int(Kd.item()) == K
        got = idx.cpu().numpy().view(np.uint32)
        assert np.array_equal(got[:K], idx_o[:K])
        assert np.all(got[K:] == 0xFFFFFFFF), "idx written beyond K"
        assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], "msg")


@pytest.mark.parametrize("n", [2, 5, 130])
def test_hybrid_exchange_streams_dense_tiles_and_lists_the_rest(B, n):
    """Exchange path 3: whole tiles that keep at least every 12th coordinate are streamed, everything else goes
    through the index list; segment cuts inside tiles, ratios on both sides of the threshold, a dense last
    tile that is not whole, unmatched workers, and runs without the optional outputs."""
    rng = np.random.default_rng(n)
    sizes = [700, 3000, 256, 1, 5000, 255, 2048, 10_000, 513, 4096, 77, 3000, 1500]
    cs = [10.0, 100.0, 1.0, 4.0, 1000.0, 12.0, 13.0, 2.0, 100.0, 11.9, 3.0, 1000.0, 5.0]
    off = synth.segment_offsets(sizes)
    N = int(off[-1]); ld = (N + 63) // 64 * 64
    peer = rand_peer(n, 7 * n + 1, singles=(1 if n % 2 else 2) if n > 3 else 0)
    for outputs in (True, False):
        r = run_round_both(B, n, N, ld, cs, off, int(rng.integers(1 << 40)), 5, peer, fused=False, outputs=outputs,
                           tuning=[(B.TUNE_EXCHANGE_PATH, 3)])
        check_round(r, N)


@pytest.mark.parametrize("n,N,ld,c", SHAPES)
@pytest.mark.parametrize("rpw", [0, 1, 2])
@pytest.mark.parametrize("with_v", [True, False])
def test_fused_round_both_wave_shapes(B, n, N, ld, c, rpw, with_v):
    """The update round either gives every wave both rows of a pair or gives each of a workgroup's two waves one
    row (they swap the tile through LDS); same bits either way, with and without the momentum buffer, with an
    unmatched worker, and in the mix-then-step order."""
    peer = rand_peer(n, n + N, singles=1 if n > 2 else 0)
    r = run_round_both(B, n, N, ld, c, None, 5, 3, peer, fused=True, with_v=with_v, tuning=[(B.TUNE_ROW_PER_WAVE, rpw)])
    check_round(r, N)


@pytest.mark.parametrize("bpc", [-1, 0, 3, 5, 9, 13, 16, 21, 32])
def test_residency_knob_changes_no_result(B, bpc):
    """The resident-workgroups knob only sizes a never-touched LDS slice: every admitted value must launch
    (a slice that the hardware refuses would surface as a HIP error) and give the oracle's bits, in every
    kernel that honours it: the three shapes of the update round, the local step, the consensus kernel."""
    n, N, ld, c = 6, 70_001, 70_144, 50.0
    peer = rand_peer(n, 11)
    for rpw in (0, 1, 2):
        for with_v in (True, False):
            r = run_round_both(B, n, N, ld, c, None, 9, 4, peer, fused=True, with_v=with_v,
                               tuning=[(B.TUNE_ROW_PER_WAVE, rpw), (B.TUNE_BLOCKS_PER_CU, bpc)])
            check_round(r, N)
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2); V0 = rand_models(n, N, ld, 3)
    for with_v in (True, False):
        Xo, Vo = X0.copy(), V0.copy()
        assert O.sgd_step(Xo, G0, Vo if with_v else None, 0.1, 0.9 if with_v else 0.0, N=N) == O.OK
        X, G, V = dev(X0), dev(G0), dev(V0)
        mean = torch.zeros(N, device="cuda"); D = torch.zeros(2, dtype=torch.float64, device="cuda")
        with B.SapsContext(n, N, ld, 0) as ctx:
            ctx.saps_set_tuning(B.TUNE_BLOCKS_PER_CU, bpc)
            ctx.saps_sgd_step(X, G, V if with_v else None, 0.1, 0.9 if with_v else 0.0)
            ctx.saps_consensus(X, mean, D[0:1])
            ctx.saps_consensus(X, None, D[1:2])
            assert ctx.saps_poll_status()[0] == 0
        assert_bits(X.cpu().numpy(), Xo, "X after the local step")
        if with_v:
            assert_bits(V.cpu().numpy(), Vo, "V after the local step")
        m_o, D_o = O.consensus(Xo, N)
        assert np.array_equal(mean.cpu().numpy().view(np.uint32), m_o.view(np.uint32))
        d = D.cpu().numpy()
        assert d[0] == d[1] and abs(d[0] - D_o) <= 1e-10 * max(D_o, 1e-30)


def test_residency_knob_rejects_values_outside_its_range(B):
    with B.SapsContext(2, 1000, 1024, 64) as ctx:
        for bad in (-2, 1, 2, 33, 1000):
            assert ctx.saps_set_tuning(B.TUNE_BLOCKS_PER_CU, bad, check=False) == B.EINVAL
        for good in (-1, 0, 3, 32):
            assert ctx.saps_set_tuning(B.TUNE_BLOCKS_PER_CU, good, check=False) == 0


@pytest.mark.parametrize("n,N,ld,c", [(4, 100_000, 100_032, 100.0), (5, 4097, 4100, 2.0), (6, 70_001, 70_144, 8.0), (3, 5, 8, 1.0)])
@pytest.mark.parametrize("xcd,nt", [(1, 1), (0, 0), (1, 0)])
def test_xcd_remap_and_plain_access_knobs_change_no_result(B, n, N, ld, c, xcd, nt):
    """Tile ranges per XCD (a permutation of the workgroups, with idle ones when the count is no multiple of 8) and
    plain instead of streaming accesses: same bits in the update round (both row orders), the tile walk, the list
    exchange, the local step and the copy."""
    tuning = [(B.TUNE_XCD_REMAP, xcd), (B.TUNE_NONTEMPORAL, nt)]
    peer = rand_peer(n, 3 * n + xcd, singles=1 if n % 2 else 0)
    for with_v in (True, False):
        for ppb in (1, 4):
            r = run_round_both(B, n, N, ld, c, None, 6, 2, peer, fused=True, with_v=with_v,
                               tuning=tuning + [(B.TUNE_PAIRS_PER_BLOCK, ppb)])
            check_round(r, N)
    for path in (1, 2):
        r = run_round_both(B, n, N, ld, c, None, 6, 2, peer, fused=False, tuning=tuning + [(B.TUNE_EXCHANGE_PATH, path)])
        check_round(r, N)
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2); V0 = rand_models(n, N, ld, 3)
    Xo, Vo = X0.copy(), V0.copy()
    assert O.sgd_step(Xo, G0, Vo, 0.1, 0.9, N=N) == O.OK
    X, G, V = dev(X0), dev(G0), dev(V0)
    dst = torch.zeros_like(X)
    with B.SapsContext(n, N, ld, 0) as ctx:
        for k, v in tuning:
            ctx.saps_set_tuning(k, v)
        ctx.saps_sgd_step(X, G, V, 0.1, 0.9)
        ctx.saps_stream_copy(dst, X)
        assert ctx.saps_poll_status()[0] == 0
    assert_bits(X.cpu().numpy(), Xo, "X"); assert_bits(V.cpu().numpy(), Vo, "V")
    assert_bits(dst.cpu().numpy(), X.cpu().numpy(), "copy")


def test_unfused_compact_and_merge_with_both_store_policies(B):
    """saps_mask_compact + saps_merge on a layout whose touched lines fit the caches (write-back scatter) and on
    one far beyond (streaming scatter): idx, msg and X as the oracle's, with an unmatched worker."""
    for n, N, c in ((5, 300_000, 50.0), (65, 2_500_000, 20.0)):
        ld = (N + 255) // 256 * 256
        cap = int(N / c * 1.2) // 4 * 4
        X0 = rand_models(n, N, ld, 21)
        peer = rand_peer(n, 8, singles=1)
        Xo = X0.copy()
        rc, K, idx_o, msg_o = O.mask_compact(Xo, N, 77, 5, c, msg_ld=cap)
        assert rc == O.OK
        assert O.merge(Xo, N, peer, idx_o, msg_o, K) == O.OK
        X = dev(X0)
        idx = torch.full((cap,), -1, dtype=torch.int32, device="cuda"); msg = torch.full((n, cap), -5.0, device="cuda")
        Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
        with B.SapsContext(n, N, ld, cap, c) as ctx:
            ctx.saps_mask_compact(X, 77, 5, idx, msg, Kd)
            ctx.saps_merge(X, peer, idx, msg, Kd)
            assert ctx.saps_poll_status() == (0, K)
        assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K])
        assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], "msg")
        assert np.all(msg.cpu().numpy()[:, K:] == -5.0)
        assert_bits(X.cpu().numpy(), Xo, f"X (n={n})")


@pytest.mark.parametrize("rpw,ppb,nt", [(0, 1, 1), (0, 4, 1), (0, 8, 0), (1, 1, 0), (2, 1, 1), (2, 1, 0)])
@pytest.mark.parametrize("with_v", [True, False])
def test_mix_then_step_in_every_kernel_shape(B, rpw, ppb, nt, with_v):
    """The mix-then-step order (Eq. (7)) in every shape of the update round: both rows per wave with 1, 4 or 8
    units per workgroup, one row per wave, plain and streaming accesses, with an unmatched worker."""
    n, N, ld, c = 7, 33_333, 33_536, 6.0
    peer = rand_peer(n, 41, singles=1)
    msg_ld = (int(N / c * 1.3) + 64) // 4 * 4
    X0 = rand_models(n, N, ld, 1); G0 = rand_models(n, N, ld, 2, pad=555.0, scale=1e-3)
    V0 = rand_models(n, N, ld, 3, pad=333.0, scale=1e-3) if with_v else None
    mu = 0.9 if with_v else 0.0
    Xo = X0.copy(); Vo = None if V0 is None else V0.copy()
    rc, K, idx_o, msg_o = O.round_(Xo, G0, Vo, N, 0.1, mu, 5, 3, peer, c, msg_ld=msg_ld, mix_first=True)
    assert rc == O.OK
    X, G = dev(X0), dev(G0); V = None if V0 is None else dev(V0)
    idx = torch.full((msg_ld,), -1, dtype=torch.int32, device="cuda")
    msg = torch.full((n, msg_ld), -5.0, device="cuda"); Kd = torch.zeros(1, dtype=torch.int64, device="cuda")
    with B.SapsContext(n, N, ld, msg_ld, c) as ctx:
        for k, v in ((B.TUNE_ROW_PER_WAVE, rpw), (B.TUNE_PAIRS_PER_BLOCK, ppb), (B.TUNE_NONTEMPORAL, nt)):
            ctx.saps_set_tuning(k, v)
        ctx.saps_round_ex(X, G, V, 0.1, mu, 5, 3, peer, idx, msg, Kd, flags=B.ROUND_MIX_THEN_STEP)
        assert ctx.saps_poll_status() == (0, K)
    assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:K], idx_o[:K])
    assert_bits(msg.cpu().numpy()[:, :K], msg_o[:, :K], "msg")
    assert np.all(msg.cpu().numpy()[:, K:] == -5.0)
    assert_bits(X.cpu().numpy(), Xo, "X")
    if with_v:
        assert_bits(V.cpu().numpy(), Vo, "V")


def test_hybrid_exchange_with_streaming_scatter(B):
    """Path 3 on a mixed-ratio layout whose touched lines exceed the caches: dense tiles are walked, the list
    kernel skips them and scatters with streaming stores."""
    n = 64
    sizes = [300_001, 700_003, 499_996, 1_000_000]
    cs = [4.0, 100.0, 8.0, 1000.0]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    N = int(off[-1]); ld = (N + 255) // 256 * 256
    cap = (int(sum(s / c for s, c in zip(sizes, cs)) * 1.1) + 256) // 4 * 4
    for path in (3, 1):
        r = run_round_both(B, n, N, ld, cs, off, 13, 6, rand_peer(n, 9), fused=False, msg_ld=cap,
                           tuning=[(B.TUNE_EXCHANGE_PATH, path)])
        check_round(r, N)


def test_consensus_with_plain_loads(B):
    n, N, ld = 9, 50_001, 50_176
    X0 = rand_models(n, N, ld, 4)
    m_o, D_o = O.consensus(X0, N)
    X = dev(X0); mean = torch.zeros(N, device="cuda"); D = torch.zeros(1, dtype=torch.float64, device="cuda")
    with B.SapsContext(n, N, ld, 0) as ctx:
        ctx.saps_set_tuning(B.TUNE_NONTEMPORAL, 0)
        ctx.saps_consensus(X, mean, D)
        assert ctx.saps_poll_status()[0] == 0
    assert np.array_equal(mean.cpu().numpy().view(np.uint32), m_o.view(np.uint32))
    assert abs(float(D.item()) - D_o) <= 1e-10 * max(D_o, 1e-30)
