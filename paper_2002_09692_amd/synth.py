"""Seeded synthetic inputs for the SAPS-PSGD round (shapes of the paper's CNN workloads).

This module is shared by the tests, the benchmark and the CPU oracle's callers.  It
holds NO arithmetic of the method itself (no mask rule, no compaction, no averaging,
no update): only model shapes, normal draws, bandwidth matrices and peer matchings,
which are *inputs* of a round.  It depends on numpy only.

Shapes follow Sec. IV-A / Table II (flat CNN parameter vectors, 32 workers,
compression ratio c = 100) and Sec. IV-D (random symmetric bandwidth matrix).
The datasets and trained weights of the paper are not used: every value is a seeded
normal draw with an initialisation-like per-tensor scale.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "workload", "resnet20_segments", "resnet18_segments",
    "resnet50_segments", "make_models", "make_grads", "random_perfect_matching",
    "bandwidth_matrix", "bandwidth_matching", "segment_offsets", "recommended_capacity",
]


# --------------------------------------------------------------------------- shapes
def resnet20_segments() -> Tuple[List[int], List[int]]:
    """CIFAR ResNet-20 with two projection shortcuts: 20 per-layer segments
    (conv + its BN pair; the projection of a stage-opening layer is folded into
    that layer; final fc + bias).  Returns (sizes, fan_in)."""
    sizes, fan = [], []
    sizes.append(3 * 16 * 9 + 32); fan.append(27)
    c_in = 16
    for stage, w in enumerate((16, 32, 64)):
        for layer in range(6):
            s = c_in * w * 9 + 2 * w
            if stage > 0 and layer == 0:
                s += c_in * w + 2 * w          # 1x1 projection + BN
            sizes.append(s); fan.append(c_in * 9)
            c_in = w
    sizes.append(64 * 10 + 10); fan.append(64)
    # the stem above plus 18 conv layers plus fc
    assert len(sizes) == 20 and sum(sizes) == 272_474, (len(sizes), sum(sizes))
    return sizes, fan


def _conv_bn(sizes, fan, c_out, c_in, k):
    sizes += [c_out * c_in * k * k, c_out, c_out]
    fan += [c_in * k * k] * 3


def resnet18_segments() -> Tuple[List[int], List[int]]:
    """CIFAR-style ResNet-18 (3x3 stem, 10 classes): 62 parameter tensors in
    definition order (conv, BN weight, BN bias ...; fc weight, fc bias)."""
    sizes, fan = [], []
    _conv_bn(sizes, fan, 64, 3, 3)
    c_in = 64
    for stage, w in enumerate((64, 128, 256, 512)):
        for block in range(2):
            _conv_bn(sizes, fan, w, c_in, 3)
            _conv_bn(sizes, fan, w, w, 3)
            if stage > 0 and block == 0:
                _conv_bn(sizes, fan, w, c_in, 1)
            c_in = w
    sizes += [512 * 10, 10]; fan += [512, 512]
    assert len(sizes) == 62 and sum(sizes) == 11_173_962, (len(sizes), sum(sizes))
    return sizes, fan


def resnet50_segments() -> Tuple[List[int], List[int]]:
    """ImageNet ResNet-50 (7x7 stem, bottlenecks [3,4,6,3], 1000 classes): 161 tensors."""
    sizes, fan = [], []
    _conv_bn(sizes, fan, 64, 3, 7)
    c_in = 64
    for w, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for block in range(blocks):
            _conv_bn(sizes, fan, w, c_in, 1)
            _conv_bn(sizes, fan, w, w, 3)
            _conv_bn(sizes, fan, 4 * w, w, 1)
            if block == 0:
                _conv_bn(sizes, fan, 4 * w, c_in, 1)
            c_in = 4 * w
    sizes += [2048 * 1000, 1000]; fan += [2048, 2048]
    assert len(sizes) == 161 and sum(sizes) == 25_557_032, (len(sizes), sum(sizes))
    return sizes, fan


def segment_offsets(sizes: Sequence[int]) -> np.ndarray:
    off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(np.asarray(sizes, dtype=np.int64), out=off[1:])
    return off


# ------------------------------------------------------------------------ workloads
@dataclasses.dataclass
class Workload:
    name: str
    n: int                       # workers
    N: int                       # coordinates per model
    seg_sizes: List[int]         # parameter tensors / layer segments, sum == N
    seg_std: List[float]         # std of the normal draw per segment
    seg_c: List[float]           # compression ratio per segment
    rounds: int
    fused: bool                  # True: SGD-momentum update fused into the round
    lr: float = 0.1
    mu: float = 0.9
    grad_std: float = 1e-3
    matching: str = "random"     # "random" | "bandwidth"
    matching_seed: int = 0
    x_seed: int = 1
    g_seed: int = 2

    @property
    def has_buffer(self) -> bool:
        """True when the round keeps a momentum buffer V (mu != 0)."""
        return self.fused and self.mu != 0.0

    @property
    def seg_off(self) -> np.ndarray:
        return segment_offsets(self.seg_sizes)

    @property
    def expected_K(self) -> float:
        return float(sum(s / c for s, c in zip(self.seg_sizes, self.seg_c)))

    @property
    def sigma_K(self) -> float:
        return float(np.sqrt(sum(s * (1 / c) * (1 - 1 / c) for s, c in zip(self.seg_sizes, self.seg_c))))

    def ld(self, align: int = 256) -> int:
        """Row stride in floats: N rounded up to whole wave tiles of 256 coordinates (1 KB), so that every
        row starts on a 1 KB boundary and a wave's 1 KB access never straddles one."""
        return (self.N + align - 1) // align * align

    B_thres: float = 50.0        # Mbps, for matching == "bandwidth"
    T_thres: int = 10            # rounds, window of recently connected edges (Alg. 3)

    def bandwidth(self) -> np.ndarray:
        """The workload's symmetric link-speed matrix (matching == "bandwidth")."""
        return bandwidth_matrix(self.n, self.matching_seed)

    def peers(self, rnd: int, selector=None) -> np.ndarray:
        """Peer permutation of round `rnd` (1-based), an involution of range(n).

        For bandwidth workloads a `selector` (an object whose saps_selector_next(rnd) returns
        (peer, info), i.e. the library's Alg. 3 peer selection created on self.bandwidth() with
        B_thres / T_thres) may be passed; it is stateful, so rounds must then be asked for in
        order.  Without one, a stateless randomised greedy matcher stands in."""
        if self.matching == "random":
            rng = np.random.default_rng([self.matching_seed, rnd])
            return random_perfect_matching(self.n, rng)
        if selector is not None:
            return np.asarray(selector.saps_selector_next(rnd)[0], dtype=np.int32)
        rng = np.random.default_rng([self.matching_seed, 7, rnd])
        return bandwidth_matching(self.bandwidth(), self.B_thres, rng)


def _kaiming(fan: Sequence[int]) -> List[float]:
    return [float(np.sqrt(2.0 / f)) for f in fan]


def _wl1() -> Workload:
    return Workload("cfg1_n4_100k", 4, 100_000, [100_000], [0.05], [100.0], 10, True)


def _wl2() -> Workload:
    s, f = resnet20_segments()
    return Workload("cfg2_n32_resnet20", 32, sum(s), s, _kaiming(f), [100.0] * len(s), 50, False,
                    matching="bandwidth")


def _wl3() -> Workload:
    s, f = resnet18_segments()
    return Workload("cfg3_n32_resnet18", 32, sum(s), s, _kaiming(f), [100.0] * len(s), 20, True)


def _wl4() -> Workload:
    s, f = resnet50_segments()
    return Workload("cfg4_n32_resnet50_c1000", 32, sum(s), s, _kaiming(f), [1000.0] * len(s), 20, False)


def _wl5() -> Workload:
    s, f = resnet18_segments()
    rng = np.random.default_rng(5)
    c = rng.choice(np.array([10.0, 100.0, 1000.0]), size=len(s)).tolist()
    return Workload("cfg5_n128_resnet18_mixedc", 128, sum(s), s, _kaiming(f), c, 10, False,
                    matching="bandwidth")


def _wl_mnist_cnn() -> Workload:
    # Table II: MNIST-CNN, 6,653,628 parameters, LR 0.05, plain SGD (the paper has no momentum), 32 workers, c = 100
    return Workload("mnist_cnn_n32", 32, 6_653_628, [6_653_628], [0.05], [100.0], 20, True, lr=0.05, mu=0.0)


def _wl_cifar10_cnn() -> Workload:
    # Table II: CIFAR10-CNN, 7,025,886 parameters, LR 0.04, plain SGD, 32 workers, c = 100
    return Workload("cifar10_cnn_n32", 32, 7_025_886, [7_025_886], [0.05], [100.0], 20, True, lr=0.04, mu=0.0)


WORKLOADS = {"cfg1": _wl1, "cfg2": _wl2, "cfg3": _wl3, "cfg4": _wl4, "cfg5": _wl5,
             "mnist_cnn": _wl_mnist_cnn, "cifar10_cnn": _wl_cifar10_cnn}


def workload(name: str) -> Workload:
    return WORKLOADS[name]()


# --------------------------------------------------------------------------- values
def _fill_rows(out: np.ndarray, N: int, seg_off: np.ndarray, seg_std: Sequence[float],
               seed: Sequence[int]) -> None:
    """Row i of out[:, :N] gets independent N(0, std_seg^2) draws; padding stays as is.
    Every row has its own generator seeded by (seed..., i), so the result does not depend
    on how the rows are spread over threads."""
    stdvec = np.repeat(np.asarray(seg_std, dtype=np.float32), np.diff(seg_off)) if len(seg_std) > 1 else None

    def one(i: int) -> None:
        rng = np.random.default_rng(list(seed) + [i])
        row = out[i, :N]
        rng.standard_normal(N, dtype=np.float32, out=row)
        if stdvec is not None:
            row *= stdvec
        else:
            row *= np.float32(seg_std[0])

    workers = min(8, os.cpu_count() or 1, out.shape[0])
    if workers > 1 and out.shape[0] * N > (1 << 22):
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(one, range(out.shape[0])))
    else:
        for i in range(out.shape[0]):
            one(i)


def make_models(wl: Workload, ld: Optional[int] = None, pad_value: float = 0.0,
                n: Optional[int] = None) -> np.ndarray:
    """n x ld fp32 matrix, row = worker (independent rows), columns [N, ld) = pad_value."""
    ld = wl.ld() if ld is None else ld
    n = wl.n if n is None else n
    X = np.full((n, ld), pad_value, dtype=np.float32)
    _fill_rows(X, wl.N, wl.seg_off, wl.seg_std, [wl.x_seed])
    return X


def make_grads(wl: Workload, rnd: int = 0, ld: Optional[int] = None, pad_value: float = 0.0,
               n: Optional[int] = None) -> np.ndarray:
    """Synthetic stochastic gradients ~ N(0, grad_std^2), one draw per (round tag, worker)."""
    ld = wl.ld() if ld is None else ld
    n = wl.n if n is None else n
    G = np.full((n, ld), pad_value, dtype=np.float32)
    _fill_rows(G, wl.N, np.array([0, wl.N]), [wl.grad_std], [wl.g_seed, rnd])
    return G


# ------------------------------------------------------------------------ matchings
def random_perfect_matching(n: int, rng: np.random.Generator) -> np.ndarray:
    """Uniformly random perfect matching as a peer permutation (odd n: one self-pair)."""
    perm = rng.permutation(n)
    peer = np.arange(n, dtype=np.int32)
    for a in range(0, n - 1, 2):
        i, j = int(perm[a]), int(perm[a + 1])
        peer[i], peer[j] = j, i
    return peer


def bandwidth_matrix(n: int, seed: int, lo: float = 1.0, hi: float = 100.0) -> np.ndarray:
    """Symmetric n x n link speeds (Mbps), upper triangle U(lo, hi), B_ij = B_ji (Sec. II-C)."""
    rng = np.random.default_rng([seed, 11])
    U = rng.uniform(lo, hi, size=(n, n))
    B = np.triu(U, 1)
    B = B + B.T
    return B


def bandwidth_matching(B: np.ndarray, B_thres: float, rng: np.random.Generator) -> np.ndarray:
    """Randomised greedy matching on links with B_ij >= B_thres, then random pairing of
    whoever is left ignoring bandwidth (the two matching passes of Alg. 3, with a greedy
    matcher standing in for the maximum matching).  Only validity is guaranteed."""
    n = B.shape[0]
    peer = np.arange(n, dtype=np.int32)
    iu, ju = np.triu_indices(n, 1)
    ok = B[iu, ju] >= B_thres
    edges = np.stack([iu[ok], ju[ok]], axis=1)
    rng.shuffle(edges, axis=0)
    free = np.ones(n, dtype=bool)
    for i, j in edges:
        if free[i] and free[j]:
            peer[i], peer[j] = j, i
            free[i] = free[j] = False
    rest = np.flatnonzero(free)
    rng.shuffle(rest)
    for a in range(0, len(rest) - 1, 2):
        i, j = int(rest[a]), int(rest[a + 1])
        peer[i], peer[j] = j, i
    return peer


def recommended_capacity(wl: Workload) -> int:
    """Message capacity per row: E[K] + 8 sigma + 64, rounded up to a multiple of 4."""
    cap = int(np.ceil(wl.expected_K + 8.0 * wl.sigma_K)) + 64
    cap = min(cap, wl.N)
    return (cap + 3) // 4 * 4
