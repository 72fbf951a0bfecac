"""ctypes loader for the CPU oracle (oracle/saps_oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this; the
GPU library never does, and this module imports nothing of the GPU package.
Every function works in place on C-contiguous numpy arrays and mirrors one C entry.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "saps_oracle.cpp")
_LIB = os.path.join(_HERE, "libsaps_oracle.so")
# The test of the pins themselves points this at a deliberately broken build of the oracle.  A stray
# variable must never swap the checker under the other tests, so the override is refused unless that
# test's own marker variable is set as well.
_OVERRIDE = os.environ.get("SAPS_ORACLE_LIB")
if _OVERRIDE and os.environ.get("SAPS_ORACLE_MUTATION_RUN") != "1":
    raise RuntimeError("SAPS_ORACLE_LIB is set but SAPS_ORACLE_MUTATION_RUN != 1: refusing to replace the oracle "
                       "(only tests/test_oracle_pins_catch_mistakes.py may do that)")

OK, EINVAL, EMATCH, ECAPACITY = 0, 1, 2, 3

CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-mfma", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (single translation unit, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["g++", *CXXFLAGS, _SRC, "-o", tmp], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(_OVERRIDE if _OVERRIDE else build())
        vp, i32, i64, u64, f32, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_double
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]; L.oracle_philox4x32_10.restype = None
        L.oracle_threshold.argtypes = [f64]; L.oracle_threshold.restype = u64
        L.oracle_coord_bits.argtypes = [u64, u64, i64]; L.oracle_coord_bits.restype = C.c_uint32
        L.oracle_mask.argtypes = [i64, i32, vp, vp, u64, u64, vp]; L.oracle_mask.restype = C.c_int
        L.oracle_sgd_step.argtypes = [i32, i64, i64, vp, vp, vp, f32, f32]; L.oracle_sgd_step.restype = C.c_int
        L.oracle_mask_compact.argtypes = [i32, i64, i64, i32, vp, vp, vp, u64, u64, vp, vp, i64, vp]
        L.oracle_mask_compact.restype = C.c_int
        L.oracle_merge.argtypes = [i32, i64, i64, vp, vp, vp, vp, i64, i64]; L.oracle_merge.restype = C.c_int
        L.oracle_round.argtypes = [i32, i64, i64, i32, vp, vp, vp, vp, vp, f32, f32, u64, u64, vp, vp, vp, i64, vp]
        L.oracle_round.restype = C.c_int
        L.oracle_round_mix_then_step.argtypes = L.oracle_round.argtypes; L.oracle_round_mix_then_step.restype = C.c_int
        L.oracle_consensus.argtypes = [i32, i64, i64, vp, vp, vp]; L.oracle_consensus.restype = C.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a: np.ndarray, dtype, name: str) -> np.ndarray:
    if a.dtype != dtype or not a.flags.c_contiguous:
        raise TypeError(f"{name}: need C-contiguous {np.dtype(dtype)}")
    return a


def _segs(N: int, seg_off, seg_c) -> Tuple[np.ndarray, np.ndarray]:
    if seg_off is None:
        seg_off = [0, N]
    so = np.ascontiguousarray(seg_off, dtype=np.int64)
    sc = np.ascontiguousarray(np.broadcast_to(np.asarray(seg_c, dtype=np.float64), (len(so) - 1,)))
    return so, sc


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    c = np.asarray(ctr, dtype=np.uint32); k = np.asarray(key, dtype=np.uint32); o = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c), _p(k), _p(o))
    return tuple(int(v) for v in o)


def threshold(c: float) -> int:
    return int(lib().oracle_threshold(float(c)))


def coord_bits(seed: int, rnd: int, j: int) -> int:
    return int(lib().oracle_coord_bits(seed, rnd, j))


def mask(N: int, seed: int, rnd: int, seg_c, seg_off=None) -> np.ndarray:
    so, sc = _segs(N, seg_off, seg_c)
    keep = np.zeros(N, dtype=np.uint8)
    rc = lib().oracle_mask(N, len(sc), _p(so), _p(sc), seed, rnd, _p(keep))
    if rc:
        raise ValueError(f"oracle_mask rc={rc}")
    return keep


def sgd_step(X: np.ndarray, G: np.ndarray, V: Optional[np.ndarray], lr: float, mu: float, N: Optional[int] = None) -> int:
    _chk(X, np.float32, "X"); _chk(G, np.float32, "G")
    if V is not None:
        _chk(V, np.float32, "V")
    n, ld = X.shape
    N = ld if N is None else N
    return lib().oracle_sgd_step(n, N, ld, _p(X), _p(G), _p(V), lr, mu)


def mask_compact(X: np.ndarray, N: int, seed: int, rnd: int, seg_c, seg_off=None, msg_ld: Optional[int] = None):
    """Returns (rc, K, idx[msg_ld] u32, msg[n, msg_ld] f32)."""
    _chk(X, np.float32, "X")
    n, ld = X.shape
    so, sc = _segs(N, seg_off, seg_c)
    msg_ld = N if msg_ld is None else msg_ld
    idx = np.zeros(msg_ld, dtype=np.uint32)
    msg = np.zeros((n, msg_ld), dtype=np.float32)
    K = np.zeros(1, dtype=np.int64)
    rc = lib().oracle_mask_compact(n, N, ld, len(sc), _p(so), _p(sc), _p(X), seed, rnd, _p(idx), _p(msg), msg_ld, _p(K))
    return rc, int(K[0]), idx, msg


def merge(X: np.ndarray, N: int, peer: np.ndarray, idx: np.ndarray, msg: np.ndarray, K: int) -> int:
    _chk(X, np.float32, "X"); _chk(idx, np.uint32, "idx"); _chk(msg, np.float32, "msg")
    peer = np.ascontiguousarray(peer, dtype=np.int32)
    n, ld = X.shape
    return lib().oracle_merge(n, N, ld, _p(X), _p(peer), _p(idx), _p(msg), msg.shape[1], K)


def round_(X: np.ndarray, G: Optional[np.ndarray], V: Optional[np.ndarray], N: int, lr: float, mu: float,
           seed: int, rnd: int, peer: np.ndarray, seg_c, seg_off=None, msg_ld: Optional[int] = None, mix_first: bool = False):
    """One round in place on X (and V), in Alg. 2 order or (mix_first=True) in the order of the
    recursion of Sec. III, Eq. (7): exchange the models of the start of the round, then step.
    Returns (rc, K, idx, msg)."""
    _chk(X, np.float32, "X")
    if G is not None:
        _chk(G, np.float32, "G")
    if V is not None:
        _chk(V, np.float32, "V")
    n, ld = X.shape
    so, sc = _segs(N, seg_off, seg_c)
    peer = np.ascontiguousarray(peer, dtype=np.int32)
    msg_ld = N if msg_ld is None else msg_ld
    idx = np.zeros(msg_ld, dtype=np.uint32)
    msg = np.zeros((n, msg_ld), dtype=np.float32)
    K = np.zeros(1, dtype=np.int64)
    fn = lib().oracle_round_mix_then_step if mix_first else lib().oracle_round
    rc = fn(n, N, ld, len(sc), _p(so), _p(sc), _p(X), _p(G), _p(V), lr, mu, seed, rnd,
            _p(peer), _p(idx), _p(msg), msg_ld, _p(K))
    return rc, int(K[0]), idx, msg


def consensus(X: np.ndarray, N: Optional[int] = None):
    """Returns (mean fp32[N], D) = average model and sum_i ||x_i - mean||^2."""
    _chk(X, np.float32, "X")
    n, ld = X.shape
    N = ld if N is None else N
    mean = np.zeros(N, dtype=np.float32)
    D = np.zeros(1, dtype=np.float64)
    rc = lib().oracle_consensus(n, N, ld, _p(X), _p(mean), _p(D))
    if rc:
        raise ValueError(f"oracle_consensus rc={rc}")
    return mean, float(D[0])
