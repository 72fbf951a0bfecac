"""The C-ABI library loads without a GPU and exports every function include/saps.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    """Every function declared in include/*.h (comments stripped)."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(saps_[a-zA-Z_0-9]+)\s*\(", text))
    return sorted(names)


def _lib():
    from paper_2002_09692_amd import build
    if not os.path.exists(build.LIB):
        build.build(force=True)            # nothing built yet: compile once (hipcc cross-compiles without a GPU)
    return ctypes.CDLL(build.LIB)


def test_header_declares_the_four_entry_points():
    names = _declared()
    for must in ("saps_round", "saps_mask_compact", "saps_merge", "saps_sgd_step", "saps_create", "saps_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    L = _lib()
    for name in _declared():
        assert hasattr(L, name), name
    L.saps_abi_version.restype = ctypes.c_int32
    assert L.saps_abi_version() >= 1


def test_binding_lists_the_same_symbols():
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None:
        return
    from paper_2002_09692_amd import binding
    assert sorted(binding.EXPORTS + binding.SELECT_EXPORTS) == _declared()


def test_host_side_errors_without_a_gpu():
    # argument checks that return before any HIP call
    L = _lib()
    L.saps_create.restype = ctypes.c_int
    h = ctypes.c_void_p()
    assert L.saps_create(ctypes.byref(h), None, ctypes.c_int64(0), None) == 1
    assert L.saps_create(None, None, ctypes.c_int64(0), None) == 1
    L.saps_destroy.restype = ctypes.c_int
    assert L.saps_destroy(None) == 1
    L.saps_last_error.restype = ctypes.c_char_p
    assert L.saps_last_error(None) == b""                   # no context: the thread's last context-free error, none yet
    # the context-free entry point checks its limits before any HIP call
    i32, i64, f32, u64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_uint64, ctypes.c_void_p
    L.saps_round_static.argtypes = [i32, i64, i64, ctypes.c_double, i64, vp, vp, vp, vp, f32, f32, u64, u64, vp, vp, vp, vp]
    L.saps_round_static.restype = ctypes.c_int
    peer = (ctypes.c_int32 * 2)(1, 0)
    K = ctypes.c_int64(0)
    big = (1 << 26) + 4
    assert L.saps_round_static(2, big, big, 100.0, 64, None, None, None, None, 0.0, 0.0, 1, 1, peer, None, None, ctypes.byref(K)) == 1
    assert b"67,108,864" in L.saps_last_error(None)
    assert L.saps_round_static(2, 64, 64, 100.0, 64, None, None, None, None, 0.0, 0.0, 1, 1, peer, None, None, None) == 1
    assert b"K_dev" in L.saps_last_error(None)


def test_synthetic_workloads_have_the_stated_shapes():
    from paper_2002_09692_amd import synth
    import numpy as np
    sizes = {"cfg1": (4, 100_000, 1), "cfg2": (32, 272_474, 20), "cfg3": (32, 11_173_962, 62),
             "cfg4": (32, 25_557_032, 161), "cfg5": (128, 11_173_962, 62)}
    for name, (n, N, segs) in sizes.items():
        wl = synth.workload(name)
        assert (wl.n, wl.N, len(wl.seg_sizes)) == (n, N, segs)
        assert wl.seg_off[-1] == N and wl.ld() % 64 == 0 and wl.ld() >= N
        for t in (1, 2, 3):
            p = wl.peers(t)
            assert np.array_equal(p[p], np.arange(n)) and (p != np.arange(n)).all()
        assert synth.recommended_capacity(wl) % 4 == 0
    assert set(synth.workload("cfg5").seg_c) == {10.0, 100.0, 1000.0}
    # rows are independent draws and reproducible
    wl = synth.workload("cfg1")
    A, B = synth.make_models(wl), synth.make_models(wl)
    assert np.array_equal(A, B) and not np.array_equal(A[0], A[1])
    assert abs(float(A[:, :wl.N].std()) - 0.05) < 1e-3
