"""Thin ctypes binding over ``libbsse.so`` -- argument marshalling only.

Function names and argument order are those of ``include/bsse.h``.  Device buffers are
``torch`` CUDA tensors (PyTorch-ROCm supplies device memory and streams, nothing else);
every numeric step runs inside the library's HIP kernels.  The library must have been
built (``python -m paper_2605_18856_amd.build``); there is no fallback of any kind.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbsse.so")

BSSE_OK, BSSE_EINVAL, BSSE_ENOTFINITE, BSSE_EOVERFLOW, BSSE_ENOMEM, BSSE_EDEVICE, BSSE_ESTATE = range(7)
BSSE_STORAGE_F32, BSSE_STORAGE_BF16 = 0, 1
BSSE_PATH_AUTO, BSSE_PATH_VALU, BSSE_PATH_MFMA, BSSE_PATH_MFMA_SPLIT = 0, 1, 2, 3

EXPORTS = [
    "bsse_create", "bsse_create_ex", "bsse_destroy", "bsse_set_stream", "bsse_lattice",
    "bsse_lattice_count", "bsse_dirichlet", "bsse_candidates", "bsse_sweep", "bsse_sweep_reset",
    "bsse_sweep_chunk", "bsse_sweep_result", "bsse_eval", "bsse_path_name", "bsse_set_timing",
    "bsse_get_timing", "bsse_last_error", "bsse_status_name", "bsse_sweep_priors",
    "bsse_profile_lp", "bsse_polish", "bsse_sweep_topk", "bsse_lattice_around",
    "bsse_dirichlet_around", "bsse_refine", "bsse_solve_realised", "bsse_sweep_dirichlet",
    "bsse_sweep_dirichlet_chunk", "bsse_sweep_best_row", "bsse_measure_ceilings",
    "bsse_measure_mixed_ceiling",
    "bsse_sweep_static",
]


class bsse_options(ctypes.Structure):
    _fields_ = [("storage", ctypes.c_int), ("path", ctypes.c_int), ("device", ctypes.c_int)]


class bsse_result(ctypes.Structure):
    _fields_ = [("best_value", ctypes.c_double), ("best_index", ctypes.c_int64),
                ("n_evals", ctypes.c_int64), ("n_tie_evals", ctypes.c_int64)]


class BsseError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{status_name(status)}: {message}")
        self.status = status


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2605_18856_amd.build` "
                          "(there is no CPU or PyTorch fallback)")
    try:
        # PyTorch-ROCm ships its own HIP runtime under the same soname; loading torch first
        # makes this library bind to that copy, so streams and pointers are shared.
        import torch  # noqa: F401
    except ImportError:      # pragma: no cover
        pass
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64
    P = ctypes.POINTER
    L.bsse_create.argtypes = [i32, i32, i32, vp, vp, vp, P(vp)]
    L.bsse_create_ex.argtypes = [i32, i32, i32, vp, vp, vp, P(bsse_options), P(vp)]
    L.bsse_destroy.argtypes = [vp]
    L.bsse_destroy.restype = None
    L.bsse_set_stream.argtypes = [vp, vp]
    L.bsse_lattice.argtypes = [vp, i32, P(i64)]
    L.bsse_lattice_count.argtypes = [i32, i32, P(i64)]
    L.bsse_dirichlet.argtypes = [vp, u64, i64, i64, vp]
    L.bsse_candidates.argtypes = [vp, P(vp), P(i64)]
    L.bsse_sweep.argtypes = [vp, vp, i64, P(bsse_result), vp]
    L.bsse_sweep_static.argtypes = [vp, vp, i64, P(bsse_result), vp]
    L.bsse_sweep_reset.argtypes = [vp]
    L.bsse_sweep_chunk.argtypes = [vp, vp, i64, i64]
    L.bsse_sweep_result.argtypes = [vp, P(bsse_result), vp]
    L.bsse_sweep_best_row.argtypes = [vp, vp]
    L.bsse_sweep_dirichlet.argtypes = [vp, u64, i64, i64, P(bsse_result), vp]
    L.bsse_sweep_dirichlet_chunk.argtypes = [vp, u64, i64, i64, i64]
    L.bsse_eval.argtypes = [vp, vp, i64, vp, vp]
    L.bsse_sweep_priors.argtypes = [vp, vp, i64, vp, i32, vp, vp]
    L.bsse_profile_lp.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, P(ctypes.c_double), P(i32)]
    L.bsse_polish.argtypes = [vp, vp, vp, P(bsse_result), vp, P(ctypes.c_double)]
    L.bsse_solve_realised.argtypes = [vp, vp, i64, i32, vp, P(ctypes.c_double), vp, P(i32), P(i32)]
    L.bsse_sweep_topk.argtypes = [vp, vp, i64, i32, vp, vp, vp, P(i32)]
    L.bsse_lattice_around.argtypes = [vp, i32, vp, ctypes.c_float, P(i64)]
    L.bsse_refine.argtypes = [vp, i32, i32, i32, i64, u64, ctypes.c_float, ctypes.c_float, vp,
                              P(bsse_result), vp]
    L.bsse_dirichlet_around.argtypes = [vp, u64, i64, i64, vp, ctypes.c_float, vp]
    L.bsse_path_name.argtypes = [vp]
    L.bsse_path_name.restype = ctypes.c_char_p
    L.bsse_set_timing.argtypes = [vp, i32]
    L.bsse_get_timing.argtypes = [vp, P(ctypes.c_double), P(i64)]
    L.bsse_measure_ceilings.argtypes = [i32, P(ctypes.c_double), P(ctypes.c_double), P(ctypes.c_double),
                                        P(ctypes.c_double)]
    L.bsse_measure_mixed_ceiling.argtypes = [i32, i32, i32, P(ctypes.c_double)]
    L.bsse_last_error.argtypes = []
    L.bsse_last_error.restype = ctypes.c_char_p
    L.bsse_status_name.argtypes = [i32]
    L.bsse_status_name.restype = ctypes.c_char_p
    for name in EXPORTS:
        getattr(L, name)          # AttributeError here means a declared symbol is missing
    _lib = L
    return L


def status_name(status: int) -> str:
    return lib().bsse_status_name(int(status)).decode()


def bsse_last_error() -> str:
    return lib().bsse_last_error().decode()


def _check(status):
    if status != BSSE_OK:
        raise BsseError(status, bsse_last_error())


def _host_f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and a.shape != shape:
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _dev_ptr(t, dtype_name, min_elems):
    """Raw device pointer of a torch CUDA tensor after layout checks (None -> NULL)."""
    if t is None:
        return None
    import torch
    want = {"float32": torch.float32, "int32": torch.int32}[dtype_name]
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == want and t.is_contiguous()):
        raise TypeError(f"expected a contiguous CUDA {dtype_name} tensor")
    if t.numel() < min_elems:
        raise ValueError(f"tensor holds {t.numel()} elements, {min_elems} needed")
    return ctypes.c_void_p(t.data_ptr())


@dataclass
class SweepOutcome:
    best_value: float
    best_index: int
    best_response: Optional[np.ndarray]   # int32[K]; None when nothing was swept
    n_evals: int
    n_tie_evals: int


class Game:
    """Owner of one ``bsse_game*`` (released on ``close()`` / garbage collection)."""

    def __init__(self, handle, m, n, K):
        self._h = handle
        self.m, self.n, self.K = m, n, K

    @property
    def handle(self):
        if not self._h:
            raise BsseError(BSSE_ESTATE, "game is closed")
        return self._h

    def close(self):
        if self._h:
            lib().bsse_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def bsse_create(m, n, K, A, B, prior, storage=BSSE_STORAGE_F32, path=BSSE_PATH_AUTO,
                device=-1) -> Game:
    """A, B: host float32 [K][m][n]; prior: host float32 [K].  Uses the current torch stream."""
    A = _host_f32(A, (K, m, n))
    B = _host_f32(B, (K, m, n))
    prior = _host_f32(prior, (K,))
    opt = bsse_options(int(storage), int(path), int(device))
    h = ctypes.c_void_p()
    _check(lib().bsse_create_ex(m, n, K, A.ctypes.data, B.ctypes.data, prior.ctypes.data,
                                ctypes.byref(opt), ctypes.byref(h)))
    g = Game(h, m, n, K)
    try:
        import torch
        if torch.cuda.is_available():
            bsse_set_stream(g, torch.cuda.current_stream().cuda_stream)
    except ImportError:      # pragma: no cover
        pass
    return g


def bsse_destroy(g: Game):
    g.close()


def bsse_set_stream(g: Game, hip_stream: int):
    _check(lib().bsse_set_stream(g.handle, ctypes.c_void_p(hip_stream)))


def bsse_path_name(g: Game) -> str:
    return lib().bsse_path_name(g.handle).decode()


def bsse_lattice_count(m: int, N: int) -> int:
    c = ctypes.c_int64()
    _check(lib().bsse_lattice_count(m, N, ctypes.byref(c)))
    return c.value


def bsse_lattice(g: Game, N: int) -> int:
    c = ctypes.c_int64()
    _check(lib().bsse_lattice(g.handle, N, ctypes.byref(c)))
    return c.value


def bsse_dirichlet(g: Game, seed: int, first: int, count: int, out=None):
    """out: CUDA float32 tensor of >= count*m elements, or None for the handle-owned buffer."""
    _check(lib().bsse_dirichlet(g.handle, ctypes.c_uint64(seed), first, count,
                                _dev_ptr(out, "float32", count * g.m)))


def _centre(g, centre):
    c = np.ascontiguousarray(centre, dtype=np.float32)
    if c.shape != (g.m,):
        raise ValueError(f"centre must be [{g.m}]")
    return c


def bsse_lattice_around(g: Game, N: int, centre, radius: float) -> int:
    c, ctr = ctypes.c_int64(), _centre(g, centre)
    _check(lib().bsse_lattice_around(g.handle, N, ctr.ctypes.data, float(radius), ctypes.byref(c)))
    return c.value


def bsse_dirichlet_around(g: Game, seed: int, first: int, count: int, centre, radius: float, out=None):
    ctr = _centre(g, centre)
    _check(lib().bsse_dirichlet_around(g.handle, ctypes.c_uint64(seed), first, count, ctr.ctypes.data,
                                       float(radius), _dev_ptr(out, "float32", count * g.m)))


def bsse_candidates(g: Game):
    """(device pointer, count) of the handle-owned generated set."""
    p, c = ctypes.c_void_p(), ctypes.c_int64()
    _check(lib().bsse_candidates(g.handle, ctypes.byref(p), ctypes.byref(c)))
    return p.value, c.value


class _DeviceView:
    """Zero-copy description of library-owned device memory for torch.as_tensor."""

    def __init__(self, ptr, shape):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": "<f4",
                                         "data": (int(ptr), False), "version": 2}


def candidates_tensor(g: Game):
    """The handle-owned generated set as a CUDA float32 [count][m] tensor that aliases the
    library's buffer (valid until the next generation call on this handle)."""
    import torch
    ptr, cnt = bsse_candidates(g)
    if cnt == 0:
        return torch.empty((0, g.m), dtype=torch.float32, device="cuda")
    return torch.as_tensor(_DeviceView(ptr, (cnt, g.m)), device="cuda")


def candidates_to_host(g: Game) -> np.ndarray:
    """Copy of the handle-owned generated set as float32 [count][m]."""
    import torch
    t = candidates_tensor(g)
    torch.cuda.current_stream().synchronize()
    return t.clone().cpu().numpy()


def _outcome(g, res, br):
    has = res.best_index >= 0
    return SweepOutcome(res.best_value, res.best_index, br.copy() if has else None,
                        res.n_evals, res.n_tie_evals)


def bsse_sweep(g: Game, candidates=None, count: Optional[int] = None) -> SweepOutcome:
    """candidates: CUDA float32 [count][m] tensor, or None for the generated set."""
    if candidates is not None and count is None:
        count = candidates.numel() // g.m
    if count is None:
        count = 0
    res = bsse_result()
    br = np.full(g.K, -1, dtype=np.int32)
    _check(lib().bsse_sweep(g.handle, _dev_ptr(candidates, "float32", count * g.m), count,
                            ctypes.byref(res), br.ctypes.data))
    return _outcome(g, res, br)


def bsse_sweep_static(g: Game, candidates, count: Optional[int] = None) -> SweepOutcome:
    """bsse_sweep through the entry point that allocates nothing (explicit candidates only)."""
    if count is None:
        count = candidates.numel() // g.m
    res = bsse_result()
    br = np.full(g.K, -1, dtype=np.int32)
    _check(lib().bsse_sweep_static(g.handle, _dev_ptr(candidates, "float32", count * g.m), count,
                                   ctypes.byref(res), br.ctypes.data))
    return _outcome(g, res, br)


def bsse_sweep_priors(g: Game, priors, candidates=None, count: Optional[int] = None):
    """priors: float32 [P][K] (host); one SweepOutcome per prior."""
    pri = np.ascontiguousarray(priors, dtype=np.float32)
    if pri.ndim != 2 or pri.shape[1] != g.K:
        raise ValueError(f"priors must be [P][{g.K}]")
    P = pri.shape[0]
    if candidates is not None and count is None:
        count = candidates.numel() // g.m
    if count is None:
        count = 0
    res = (bsse_result * max(P, 1))()
    br = np.full((max(P, 1), g.K), -1, dtype=np.int32)
    _check(lib().bsse_sweep_priors(g.handle, _dev_ptr(candidates, "float32", count * g.m), count,
                                   pri.ctypes.data, P, ctypes.cast(res, ctypes.c_void_p),
                                   br.ctypes.data))
    return [_outcome(g, res[p], br[p]) for p in range(P)]


def bsse_sweep_topk(g: Game, k: int, candidates=None, count: Optional[int] = None):
    """(values float64 [f], indices int64 [f], best responses int32 [f][K]) of the f = min(k, count)
    best candidates, best first."""
    if candidates is not None and count is None:
        count = candidates.numel() // g.m
    if count is None:
        count = 0
    kk = max(int(k), 1)
    v = np.zeros(kk, dtype=np.float64)
    idx = np.full(kk, -1, dtype=np.int64)
    br = np.full((kk, g.K), -1, dtype=np.int32)
    found = ctypes.c_int(0)
    _check(lib().bsse_sweep_topk(g.handle, _dev_ptr(candidates, "float32", count * g.m), count, int(k),
                                 v.ctypes.data, idx.ctypes.data, br.ctypes.data, ctypes.byref(found)))
    f = found.value
    return v[:f].copy(), idx[:f].copy(), br[:f].copy()


def bsse_solve_realised(g: Game, candidates=None, count: Optional[int] = None, max_profiles: int = 1 << 20):
    """(value, x float32 [m], profile int32 [K], distinct profiles realised, programs solved)."""
    if candidates is not None and count is None:
        count = candidates.numel() // g.m
    if count is None:
        count = 0
    x = np.zeros(g.m, dtype=np.float32)
    prof = np.full(g.K, -1, dtype=np.int32)
    v, npf, ns = ctypes.c_double(0.0), ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().bsse_solve_realised(g.handle, _dev_ptr(candidates, "float32", count * g.m), count,
                                     int(max_profiles), x.ctypes.data, ctypes.byref(v), prof.ctypes.data,
                                     ctypes.byref(npf), ctypes.byref(ns)))
    return v.value, x, prof, npf.value, ns.value


def bsse_refine(g: Game, k: int, rounds: int, lattice_N: int = 0, cloud_count: int = 0, seed: int = 0,
                radius: float = 0.25, shrink: float = 0.25):
    """(x float32 [m], value, best responses int32 [K], evaluations spent) after `rounds` rounds of
    top-k + local re-sweep starting from the handle-owned generated set."""
    x = np.zeros(g.m, dtype=np.float32)
    br = np.full(g.K, -1, dtype=np.int32)
    res = bsse_result()
    _check(lib().bsse_refine(g.handle, int(k), int(rounds), int(lattice_N), int(cloud_count),
                             ctypes.c_uint64(seed), float(radius), float(shrink), x.ctypes.data,
                             ctypes.byref(res), br.ctypes.data))
    return x, res.best_value, br, res.n_evals


def bsse_profile_lp(A, B, prior, profile):
    """Host-only: (feasible, value, x float64 [m]) of the linear program of one follower profile."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    pr = np.ascontiguousarray(prior, dtype=np.float32)
    prof = np.ascontiguousarray(profile, dtype=np.int32)
    K, m, n = A.shape
    if B.shape != A.shape or pr.shape != (K,) or prof.shape != (K,):
        raise ValueError("A, B: [K][m][n]; prior, profile: [K]")
    x = np.zeros(m, dtype=np.float64)
    v, ok = ctypes.c_double(0.0), ctypes.c_int(0)
    _check(lib().bsse_profile_lp(m, n, K, A.ctypes.data, B.ctypes.data, pr.ctypes.data,
                                 prof.ctypes.data, x.ctypes.data, ctypes.byref(v), ctypes.byref(ok)))
    return bool(ok.value), (v.value if ok.value else None), (x if ok.value else None)


@dataclass
class PolishOutcome:
    x: np.ndarray                  # float32 [m]: the polished commitment
    value: float                   # its V as the sweep kernels compute it
    point: int                     # 0 = the program's vertex ... 7 = the sweep's own winner
    best_response: np.ndarray      # int32 [K]
    lp_value: float                # optimum of the profile's linear program


def bsse_polish(g: Game, profile=None) -> PolishOutcome:
    prof = None if profile is None else np.ascontiguousarray(profile, dtype=np.int32)
    if prof is not None and prof.shape != (g.K,):
        raise ValueError(f"profile must be [{g.K}]")
    x = np.zeros(g.m, dtype=np.float32)
    br = np.full(g.K, -1, dtype=np.int32)
    res, lp = bsse_result(), ctypes.c_double(0.0)
    _check(lib().bsse_polish(g.handle, None if prof is None else prof.ctypes.data, x.ctypes.data,
                             ctypes.byref(res), br.ctypes.data, ctypes.byref(lp)))
    return PolishOutcome(x, res.best_value, int(res.best_index), br, lp.value)


def bsse_sweep_reset(g: Game):
    _check(lib().bsse_sweep_reset(g.handle))


def bsse_sweep_chunk(g: Game, candidates, count: int, index_base: int):
    _check(lib().bsse_sweep_chunk(g.handle, _dev_ptr(candidates, "float32", count * g.m), count,
                                  index_base))


def bsse_sweep_best_row(g: Game) -> np.ndarray:
    x = np.empty(g.m, dtype=np.float32)
    _check(lib().bsse_sweep_best_row(g.handle, x.ctypes.data))
    return x


def bsse_sweep_dirichlet(g: Game, seed: int, first: int, count: int) -> SweepOutcome:
    res = bsse_result()
    br = np.full(g.K, -1, dtype=np.int32)
    _check(lib().bsse_sweep_dirichlet(g.handle, seed, first, count, ctypes.byref(res), br.ctypes.data))
    return _outcome(g, res, br)


def bsse_sweep_dirichlet_chunk(g: Game, seed: int, first: int, count: int, index_base: int):
    _check(lib().bsse_sweep_dirichlet_chunk(g.handle, seed, first, count, index_base))


def bsse_sweep_result(g: Game) -> SweepOutcome:
    res = bsse_result()
    br = np.full(g.K, -1, dtype=np.int32)
    _check(lib().bsse_sweep_result(g.handle, ctypes.byref(res), br.ctypes.data))
    return _outcome(g, res, br)


def bsse_eval(g: Game, candidates, count: int, values_out=None, br_out=None):
    """values_out: CUDA float32 [count]; br_out: CUDA int32 [count][K]; either may be None."""
    _check(lib().bsse_eval(g.handle, _dev_ptr(candidates, "float32", count * g.m), count,
                           _dev_ptr(values_out, "float32", count),
                           _dev_ptr(br_out, "int32", count * g.K)))


def bsse_set_timing(g: Game, enabled: bool):
    _check(lib().bsse_set_timing(g.handle, int(bool(enabled))))


def bsse_get_timing(g: Game):
    ms, n = ctypes.c_double(), ctypes.c_int64()
    _check(lib().bsse_get_timing(g.handle, ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def bsse_ceilings(device: int = -1) -> dict:
    """What plain kernels reach on the device (see bsse_measure_ceilings)."""
    d = [ctypes.c_double() for _ in range(4)]
    st = lib().bsse_measure_ceilings(int(device), *[ctypes.byref(x) for x in d])
    if st != BSSE_OK:
        raise BsseError(st, "bsse_measure_ceilings failed")
    return {"stream_read_GBs": d[0].value, "mfma_bf16_TFLOPs": d[1].value,
            "mfma_f32_TFLOPs": d[2].value, "empty_launch_us": d[3].value}


def bsse_mixed_ceiling(mfma_per_round: int, valu_per_round: int, device: int = -1) -> float:
    """bf16 matrix-core TFLOP/s under a given mix of matrix and vector instructions (see
    bsse_measure_mixed_ceiling)."""
    d = ctypes.c_double()
    st = lib().bsse_measure_mixed_ceiling(int(device), int(mfma_per_round), int(valu_per_round), ctypes.byref(d))
    if st != BSSE_OK:
        raise BsseError(st, "bsse_measure_mixed_ceiling failed")
    return d.value
