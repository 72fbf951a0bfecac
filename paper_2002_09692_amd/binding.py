"""Thin ctypes binding of include/saps.h.  Argument marshalling only: every step of the
round runs in the HIP kernels of libsaps.so.  PyTorch supplies device memory and streams.

There is no CPU fallback: if the library is missing or cannot be loaded, importing the
entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch  # loaded first so that libsaps.so binds to the HIP runtime torch already mapped

from .build import LIB

OK, EINVAL, EMATCH, ECAPACITY, EHIP = 0, 1, 2, 3, 4
ROUND_MIX_THEN_STEP = 1
TUNE_PAIRS_PER_BLOCK, TUNE_XCD_REMAP, TUNE_NONTEMPORAL, TUNE_EXCHANGE_PATH, TUNE_BLOCKS_PER_CU, TUNE_PREPARE_NEXT, TUNE_ROW_PER_WAVE = 0, 1, 2, 3, 4, 5, 6
_NAMES = {OK: "SAPS_OK", EINVAL: "SAPS_EINVAL", EMATCH: "SAPS_EMATCH", ECAPACITY: "SAPS_ECAPACITY", EHIP: "SAPS_EHIP"}

EXPORTS = ("saps_abi_version", "saps_create", "saps_destroy", "saps_sgd_step", "saps_mask_compact", "saps_merge",
           "saps_round", "saps_poll_status", "saps_last_error", "saps_set_tuning", "saps_stream_copy",
           "saps_profile_enable", "saps_profile_read", "saps_consensus", "saps_round_ex", "saps_round_static",
           "saps_list_probe")


class SapsError(RuntimeError):
    def __init__(self, status: int, text: str = ""):
        super().__init__(f"{_NAMES.get(status, status)}: {text}")
        self.status = status


class _Layout(C.Structure):
    _fields_ = [("n", C.c_int32), ("N", C.c_int64), ("ld", C.c_int64), ("n_seg", C.c_int32),
                ("seg_off", C.POINTER(C.c_int64)), ("seg_c", C.POINTER(C.c_double))]


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree libsaps.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB):
        raise ImportError(f"{LIB} not found: run `python -c 'import __graft_entry__ as g; g.build()'` first "
                          "(there is no fallback path)")
    L = C.CDLL(LIB)
    vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
    L.saps_abi_version.argtypes = []; L.saps_abi_version.restype = i32
    L.saps_create.argtypes = [C.POINTER(vp), C.POINTER(_Layout), i64, vp]; L.saps_create.restype = C.c_int
    L.saps_destroy.argtypes = [vp]; L.saps_destroy.restype = C.c_int
    L.saps_sgd_step.argtypes = [vp, vp, vp, vp, f32, f32]; L.saps_sgd_step.restype = C.c_int
    L.saps_mask_compact.argtypes = [vp, vp, u64, u64, vp, vp, vp]; L.saps_mask_compact.restype = C.c_int
    L.saps_merge.argtypes = [vp, vp, vp, vp, vp, vp]; L.saps_merge.restype = C.c_int
    L.saps_round.argtypes = [vp, vp, vp, vp, f32, f32, u64, u64, vp, vp, vp, vp]; L.saps_round.restype = C.c_int
    L.saps_poll_status.argtypes = [vp, C.POINTER(i64)]; L.saps_poll_status.restype = C.c_int
    L.saps_last_error.argtypes = [vp]; L.saps_last_error.restype = C.c_char_p
    L.saps_set_tuning.argtypes = [vp, i32, i32]; L.saps_set_tuning.restype = C.c_int
    L.saps_stream_copy.argtypes = [vp, vp, vp, i64]; L.saps_stream_copy.restype = C.c_int
    L.saps_round_ex.argtypes = [vp, vp, vp, vp, f32, f32, u64, u64, vp, vp, vp, vp, C.c_uint32]; L.saps_round_ex.restype = C.c_int
    L.saps_consensus.argtypes = [vp, vp, vp, vp]; L.saps_consensus.restype = C.c_int
    L.saps_round_static.argtypes = [i32, i64, i64, C.c_double, i64, vp, vp, vp, vp, f32, f32, u64, u64, vp, vp, vp, vp]
    L.saps_round_static.restype = C.c_int
    L.saps_list_probe.argtypes = [vp, vp, vp, vp, i32]; L.saps_list_probe.restype = C.c_int
    L.saps_profile_enable.argtypes = [vp, i32]; L.saps_profile_enable.restype = C.c_int
    L.saps_profile_read.argtypes = [vp, C.POINTER(i32), C.POINTER(C.c_double)]; L.saps_profile_read.restype = C.c_int
    _lib = L
    return L


def _dev(t: Optional[torch.Tensor], dtype, name: str):
    """Raw device pointer of a contiguous device tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous device tensor of {dtype}")
    return C.c_void_p(t.data_ptr())


def _peer(peer) -> np.ndarray:
    if isinstance(peer, torch.Tensor):
        peer = peer.cpu().numpy()
    return np.ascontiguousarray(peer, dtype=np.int32)


class _SelectInfo(C.Structure):
    _fields_ = [("rc_connected", C.c_int32), ("rc_components", C.c_int32), ("first_pairs", C.c_int32),
                ("second_pairs", C.c_int32), ("min_bandwidth", C.c_double), ("mean_bandwidth", C.c_double)]


SELECT_EXPORTS = ("saps_selector_create", "saps_selector_destroy", "saps_selector_next", "saps_selector_get_R",
                  "saps_max_matching")


class PeerSelector:
    """Host-side adaptive peer selection (include/saps_select.h): Alg. 3 round by round."""

    def __init__(self, B: np.ndarray, B_thres: float, T_thres: int, seed: int = 0):
        L = load_library()
        L.saps_selector_create.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_void_p, C.c_double, C.c_int64, C.c_uint64]
        L.saps_selector_next.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(_SelectInfo)]
        L.saps_selector_get_R.argtypes = [C.c_void_p, C.c_void_p]
        L.saps_selector_destroy.argtypes = [C.c_void_p]
        Bc = np.ascontiguousarray(B, dtype=np.float64)
        if Bc.ndim != 2 or Bc.shape[0] != Bc.shape[1]:
            raise ValueError("B: need a square matrix")
        self.n = Bc.shape[0]
        h = C.c_void_p()
        if L.saps_selector_create(C.byref(h), self.n, Bc.ctypes.data_as(C.c_void_p), B_thres, T_thres, seed) != 0:
            raise SapsError(EINVAL, "saps_selector_create")
        self._h, self._L = h, L

    def saps_selector_next(self, t: int):
        """Returns (peer[n] int32, info dict) for round t."""
        peer = np.empty(self.n, dtype=np.int32)
        info = _SelectInfo()
        if self._L.saps_selector_next(self._h, t, peer.ctypes.data_as(C.c_void_p), C.byref(info)) != 0:
            raise SapsError(EINVAL, "saps_selector_next")
        return peer, {k: getattr(info, k) for k, _ in _SelectInfo._fields_}

    def saps_selector_get_R(self) -> np.ndarray:
        R = np.empty((self.n, self.n), dtype=np.int64)
        self._L.saps_selector_get_R(self._h, R.ctypes.data_as(C.c_void_p))
        return R

    def close(self):
        if getattr(self, "_h", None):
            self._L.saps_selector_destroy(self._h)
            self._h = None

    __del__ = close


def saps_max_matching(E: np.ndarray, seed: int = 0):
    """Maximum-cardinality matching of the graph E (n x n 0/1).  Returns (pairs, peer[n])."""
    L = load_library()
    L.saps_max_matching.argtypes = [C.c_int32, C.c_void_p, C.c_uint64, C.c_void_p]
    Ec = np.ascontiguousarray(E, dtype=np.uint8)
    n = Ec.shape[0]
    peer = np.empty(n, dtype=np.int32)
    pairs = L.saps_max_matching(n, Ec.ctypes.data_as(C.c_void_p), seed, peer.ctypes.data_as(C.c_void_p))
    return int(pairs), peer


def saps_round_static(n: int, N: int, ld: int, c: float, msg_ld: int, X, G, V, lr: float, mu: float, seed: int, rnd: int,
                      peer, idx=None, msg=None, K_dev=None, stream: Optional[torch.cuda.Stream] = None, check: bool = True) -> int:
    """saps_round without a context, on the library's fixed scratch (for callers that cannot allocate)."""
    L = load_library()
    p = _peer(peer)
    if p.shape != (n,):
        raise ValueError("peer: need n entries")
    for t, name in ((X, "X"), (G, "G"), (V, "V")):
        if t is not None and tuple(t.shape) != (n, ld):
            raise ValueError(f"{name}: shape {tuple(t.shape)} != {(n, ld)}")
    if msg is not None and tuple(msg.shape) != (n, msg_ld):
        raise ValueError("msg: shape")
    if idx is not None and idx.numel() < msg_ld:
        raise ValueError("idx: fewer than msg_ld entries")
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = L.saps_round_static(n, N, ld, float(c), msg_ld, C.c_void_p(st.cuda_stream), _dev(X, torch.float32, "X"),
                             _dev(G, torch.float32, "G"), _dev(V, torch.float32, "V"), lr, mu, seed, rnd,
                             p.ctypes.data_as(C.c_void_p), _dev(idx, torch.int32, "idx"), _dev(msg, torch.float32, "msg"),
                             _dev(K_dev, torch.int64, "K_dev"))
    if check and rc != OK:
        raise SapsError(rc, L.saps_last_error(None).decode())
    return rc


class SapsContext:
    """saps_create / saps_destroy plus the per-round entry points as methods with the C names."""

    def __init__(self, n: int, N: int, ld: int, msg_ld: int, seg_c: Sequence[float] | float = 100.0,
                 seg_off: Optional[Sequence[int]] = None, stream: Optional[torch.cuda.Stream] = None):
        L = load_library()
        if seg_off is None:
            seg_off = [0, N]
        so = np.ascontiguousarray(seg_off, dtype=np.int64)
        sc = np.ascontiguousarray(np.broadcast_to(np.asarray(seg_c, dtype=np.float64), (len(so) - 1,)))
        lay = _Layout(n, N, ld, len(sc), so.ctypes.data_as(C.POINTER(C.c_int64)), sc.ctypes.data_as(C.POINTER(C.c_double)))
        self.n, self.N, self.ld, self.msg_ld = n, N, ld, msg_ld
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        rc = L.saps_create(C.byref(h), C.byref(lay), msg_ld, C.c_void_p(self.stream.cuda_stream))
        if rc != OK:
            raise SapsError(rc, "saps_create")
        self._h, self._L = h, L

    # -- lifetime
    def close(self):
        if getattr(self, "_h", None):
            self._L.saps_destroy(self._h)
            self._h = None

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _rc(self, rc: int, check: bool) -> int:
        if check and rc != OK:
            raise SapsError(rc, self._L.saps_last_error(self._h).decode())
        return rc

    def _rows(self, t: Optional[torch.Tensor], name: str):
        if t is not None and tuple(t.shape) != (self.n, self.ld):
            raise ValueError(f"{name}: shape {tuple(t.shape)} != {(self.n, self.ld)}")
        return _dev(t, torch.float32, name)

    def _msg(self, t: Optional[torch.Tensor]):
        if t is not None and tuple(t.shape) != (self.n, self.msg_ld):
            raise ValueError(f"msg: shape {tuple(t.shape)} != {(self.n, self.msg_ld)}")
        return _dev(t, torch.float32, "msg")

    def _idx(self, t: Optional[torch.Tensor]):
        if t is not None and t.numel() < self.msg_ld:
            raise ValueError("idx: fewer than msg_ld entries")
        return _dev(t, torch.int32, "idx")          # uint32 bit pattern in an int32 tensor

    @staticmethod
    def _K(t: Optional[torch.Tensor]):
        if t is not None and t.numel() < 1:
            raise ValueError("K_dev: empty")
        return _dev(t, torch.int64, "K_dev")

    # -- entry points (names of the C ABI)
    def saps_sgd_step(self, X, G, V, lr: float, mu: float, check: bool = True) -> int:
        return self._rc(self._L.saps_sgd_step(self._h, self._rows(X, "X"), self._rows(G, "G"), self._rows(V, "V"), lr, mu), check)

    def saps_mask_compact(self, X, seed: int, rnd: int, idx, msg, K_dev, check: bool = True) -> int:
        return self._rc(self._L.saps_mask_compact(self._h, self._rows(X, "X"), seed, rnd, self._idx(idx), self._msg(msg),
                                                  self._K(K_dev)), check)

    def saps_merge(self, X, peer, idx, msg, K_dev, check: bool = True) -> int:
        p = _peer(peer)
        if p.shape != (self.n,):
            raise ValueError("peer: need n entries")
        return self._rc(self._L.saps_merge(self._h, self._rows(X, "X"), p.ctypes.data_as(C.c_void_p), self._idx(idx),
                                           self._msg(msg), self._K(K_dev)), check)

    def saps_round(self, X, G, V, lr: float, mu: float, seed: int, rnd: int, peer, idx=None, msg=None, K_dev=None,
                   check: bool = True) -> int:
        p = _peer(peer)
        if p.shape != (self.n,):
            raise ValueError("peer: need n entries")
        return self._rc(self._L.saps_round(self._h, self._rows(X, "X"), self._rows(G, "G"), self._rows(V, "V"), lr, mu,
                                           seed, rnd, p.ctypes.data_as(C.c_void_p), self._idx(idx), self._msg(msg),
                                           self._K(K_dev)), check)

    def saps_poll_status(self, check: bool = False):
        """Returns (status, K) after waiting for the stream."""
        K = C.c_int64(-1)
        rc = self._L.saps_poll_status(self._h, C.byref(K))
        return self._rc(rc, check), int(K.value)

    def saps_set_tuning(self, knob: int, value: int, check: bool = True) -> int:
        return self._rc(self._L.saps_set_tuning(self._h, knob, value), check)

    def saps_stream_copy(self, dst: torch.Tensor, src: torch.Tensor, check: bool = True) -> int:
        return self._rc(self._L.saps_stream_copy(self._h, _dev(dst, torch.float32, "dst"), _dev(src, torch.float32, "src"),
                                                 src.numel()), check)

    def saps_list_probe(self, X, idx, K_dev, write_back: bool, check: bool = True) -> int:
        return self._rc(self._L.saps_list_probe(self._h, self._rows(X, "X"), self._idx(idx), self._K(K_dev),
                                                int(write_back)), check)

    def saps_profile_enable(self, on: bool) -> int:
        return self._rc(self._L.saps_profile_enable(self._h, int(on)), True)

    def saps_profile_read(self):
        """Returns (launches, total_ms) of the dominant kernels recorded since the last read."""
        cnt = C.c_int32(0); ms = C.c_double(0.0)
        self._rc(self._L.saps_profile_read(self._h, C.byref(cnt), C.byref(ms)), True)
        return int(cnt.value), float(ms.value)

    def saps_consensus(self, X, mean_out, D_dev, check: bool = True) -> int:
        if mean_out is not None and mean_out.numel() < self.N:
            raise ValueError("mean_out: fewer than N entries")
        if D_dev.numel() < 1:
            raise ValueError("D_dev: empty")
        return self._rc(self._L.saps_consensus(self._h, self._rows(X, "X"), _dev(mean_out, torch.float32, "mean_out"),
                                               _dev(D_dev, torch.float64, "D_dev")), check)

    def saps_round_ex(self, X, G, V, lr: float, mu: float, seed: int, rnd: int, peer, idx=None, msg=None, K_dev=None,
                      flags: int = 0, check: bool = True) -> int:
        p = _peer(peer)
        if p.shape != (self.n,):
            raise ValueError("peer: need n entries")
        return self._rc(self._L.saps_round_ex(self._h, self._rows(X, "X"), self._rows(G, "G"), self._rows(V, "V"), lr, mu,
                                              seed, rnd, p.ctypes.data_as(C.c_void_p), self._idx(idx), self._msg(msg),
                                              self._K(K_dev), flags), check)
