"""ctypes binding of the C oracle (test infrastructure only).

Argument marshalling only: every number comes out of ccdc_oracle.c.  The
shared object is built with gcc next to the sources; nothing here touches the
GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libccdc_oracle.so")
_SRCS = ["ccdc_oracle.c"]
_DEPS = ["ccdc_oracle.c", "ccdc_oracle.h", "ccdc_oracle_stages.inc", "ccdc_oracle_compression.inc",
         "ccdc_oracle_h16.inc"]


def build_library(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, single thread) if missing or stale."""
    stale = force or not os.path.exists(_SO)
    if not stale:
        so_time = os.path.getmtime(_SO)
        stale = any(os.path.getmtime(os.path.join(_HERE, d)) > so_time for d in _DEPS)
    if stale:
        cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared",
               "-o", _SO] + [os.path.join(_HERE, s) for s in _SRCS] + ["-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


class _CPlan(C.Structure):
    _fields_ = [
        ("K", C.c_int), ("r", C.c_int), ("Q", C.c_int), ("N", C.c_int),
        ("J", C.c_int), ("c", C.c_int), ("m", C.c_int),
        ("n_batch", C.c_int64), ("n_round", C.c_int64),
        ("batch_job", C.POINTER(C.c_int)),
        ("batch_file0", C.POINTER(C.c_int)),
        ("batch_label", C.POINTER(C.c_int)),
        ("round_member", C.POINTER(C.c_int)),
        ("round_batch", C.POINTER(C.c_int)),
    ]


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = C.CDLL(build_library())
    P = C.POINTER(_CPlan)
    lib.orc_binom.restype = C.c_int64
    lib.orc_binom.argtypes = [C.c_int, C.c_int]
    lib.orc_plan_build.restype = P
    lib.orc_plan_build.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.c_int]
    lib.orc_plan_select_rounds.restype = P
    lib.orc_plan_select_rounds.argtypes = [P, C.POINTER(C.c_int64), C.c_int64]
    lib.orc_plan_repeat.restype = P
    lib.orc_plan_repeat.argtypes = [P, C.c_int]
    lib.orc_plan_free.restype = None
    lib.orc_plan_free.argtypes = [P]
    lib.orc_segment_len.restype = C.c_int64
    lib.orc_segment_len.argtypes = [C.c_int64, C.c_int]
    lib.orc_segment_count.restype = C.c_int64
    lib.orc_segment_count.argtypes = [C.c_int64, C.c_int, C.c_int]
    lib.orc_label_rank.restype = C.c_int
    lib.orc_label_rank.argtypes = [C.c_int, C.c_int]
    lib.orc_packet_len.restype = C.c_int64
    lib.orc_packet_len.argtypes = [C.c_int64, C.c_int, C.c_int]
    lib.orc_scheduled_elems.restype = C.c_int64
    lib.orc_scheduled_elems.argtypes = [P, C.c_int64]
    vp = C.c_void_p
    for sfx in ("f64", "u32", "h32"):
        for name, nptr in (("combine", 2), ("encode", 2), ("decode", 3), ("reduce", 3), ("direct", 2)):
            if sfx == "h32" and name == "direct":
                continue
            fn = getattr(lib, f"orc_{name}_{sfx}")
            fn.restype = None
            fn.argtypes = [P, C.c_int64] + [vp] * nptr
    _lib = lib
    return lib


def _arr(ptr, shape):
    n = int(np.prod(shape))
    if n == 0:
        return np.zeros(shape, dtype=np.int32)
    return np.ctypeslib.as_array(ptr, shape=(n,)).reshape(shape).astype(np.int32, copy=True)


class OraclePlan:
    """Placement + round schedule as built by orc_plan_build (read-only copies)."""

    def __init__(self, ptr):
        self._ptr = ptr
        s = ptr.contents
        self.K, self.r, self.Q, self.N = s.K, s.r, s.Q, s.N
        self.J, self.c, self.m = s.J, s.c, s.m
        self.n_batch, self.n_round = int(s.n_batch), int(s.n_round)
        self.batch_job = _arr(s.batch_job, (self.n_batch,))
        self.batch_file0 = _arr(s.batch_file0, (self.n_batch,))
        self.batch_label = _arr(s.batch_label, (self.n_batch, self.r))
        self.round_member = _arr(s.round_member, (self.n_round, self.r + 1))
        self.round_batch = _arr(s.round_batch, (self.n_round, self.r + 1))

    def __del__(self):
        try:
            if self._ptr:
                _load().orc_plan_free(self._ptr)
                self._ptr = None
        except Exception:
            pass

    # shapes of the artefacts for value length T
    def W(self, T):
        return self.c * T

    def shapes(self, T):
        W = self.c * T
        ell = segment_len(W, self.r)
        R, r1 = self.n_round, self.r + 1
        return {"V": (self.J, self.N, self.Q, T), "Vbar": (R, r1, W), "X": (R, r1, ell),
                "D": (R, r1, W), "Phi": (self.J, self.Q, T)}


def build_plan(K, r, Q, N, schedule="single", batch_order=None, gamma=1):
    """schedule: "single" (one job, one batch per r-subset) or "paper" (J=C(K,r+1) jobs).

    batch_order: one permutation (shared) or a list of J permutations (one per job).
    gamma: the whole scheme repeated on gamma consecutive blocks of jobs (Sec. IV)."""
    lib = _load()
    sched = {"single": 0, "paper": 1}[schedule]
    order, sets = None, 0
    if batch_order is not None:
        rows = np.atleast_2d(np.asarray(batch_order, dtype=np.int32))   # one row per permutation
        sets = rows.shape[0]
        order = (C.c_int * rows.size)(*[int(v) for v in rows.ravel()])
    ptr = lib.orc_plan_build(K, r, Q, N, sched, order, sets)
    if not ptr:
        raise ValueError(f"invalid parameters K={K} r={r} Q={Q} N={N} schedule={schedule}")
    if gamma != 1:
        once = ptr
        ptr = lib.orc_plan_repeat(once, int(gamma))
        lib.orc_plan_free(once)
        if not ptr:
            raise ValueError(f"invalid repetition count gamma={gamma}")
    return OraclePlan(ptr)


def select_rounds(plan, rounds):
    """Plan with the same batches and only the listed rounds (sampling a large schedule)."""
    rounds = [int(u) for u in rounds]
    arr = (C.c_int64 * max(1, len(rounds)))(*rounds)
    ptr = _load().orc_plan_select_rounds(plan._ptr, arr, len(rounds))
    if not ptr:
        raise ValueError("bad round index")
    return OraclePlan(ptr)


def segment_len(W, r):
    return int(_load().orc_segment_len(W, r))


def segment_count(W, r, rho):
    return int(_load().orc_segment_count(W, r, rho))


def label_rank(a, b):
    return int(_load().orc_label_rank(a, b))


def packet_len(W, r, a):
    return int(_load().orc_packet_len(W, r, a))


def scheduled_elems(plan, T):
    return int(_load().orc_scheduled_elems(plan._ptr, T))


def closed_form_elems(plan, T):
    """Per round (r+1) packets of c*T/r elements each (Sec. IV-B load analysis)."""
    return Fraction((plan.r + 1) * plan.c * T, plan.r) * plan.n_round


def _mode(a):
    if a.dtype == np.uint32:
        return "u32", np.uint32
    if a.dtype in (np.float32, np.float64):
        return "f64", np.float64
    raise TypeError(f"unsupported dtype {a.dtype}")


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _check(a, dtype, shape, name):
    if a.dtype != dtype or not a.flags.c_contiguous or tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: want contiguous {np.dtype(dtype).name}{tuple(shape)}, "
                         f"got {a.dtype}{tuple(a.shape)}")


def combine(plan, T, V):
    sfx, el = _mode(V)
    sh = plan.shapes(T)
    _check(V, np.float32 if sfx == "f64" else np.uint32, sh["V"], "V")
    out = np.empty(sh["Vbar"], dtype=el)
    getattr(_load(), f"orc_combine_{sfx}")(plan._ptr, T, _ptr(V), _ptr(out))
    return out


def encode(plan, T, Vbar):
    sfx, el = _mode(Vbar)
    sh = plan.shapes(T)
    _check(Vbar, el, sh["Vbar"], "Vbar")
    out = np.empty(sh["X"], dtype=el)
    getattr(_load(), f"orc_encode_{sfx}")(plan._ptr, T, _ptr(Vbar), _ptr(out))
    return out


def decode(plan, T, X, Vbar):
    sfx, el = _mode(Vbar)
    sh = plan.shapes(T)
    _check(X, el, sh["X"], "X")
    _check(Vbar, el, sh["Vbar"], "Vbar")
    out = np.zeros(sh["D"], dtype=el)
    getattr(_load(), f"orc_decode_{sfx}")(plan._ptr, T, _ptr(X), _ptr(Vbar), _ptr(out))
    return out


def reduce(plan, T, V, D):
    sfx, el = _mode(V)
    sh = plan.shapes(T)
    _check(V, np.float32 if sfx == "f64" else np.uint32, sh["V"], "V")
    _check(D, el, sh["D"], "D")
    out = np.empty(sh["Phi"], dtype=el)
    getattr(_load(), f"orc_reduce_{sfx}")(plan._ptr, T, _ptr(V), _ptr(D), _ptr(out))
    return out


def direct(plan, T, V):
    sfx, el = _mode(V)
    sh = plan.shapes(T)
    _check(V, np.float32 if sfx == "f64" else np.uint32, sh["V"], "V")
    out = np.empty(sh["Phi"], dtype=el)
    getattr(_load(), f"orc_direct_{sfx}")(plan._ptr, T, _ptr(V), _ptr(out))
    return out


class _CCPlan(C.Structure):
    _fields_ = [
        ("K", C.c_int), ("r", C.c_int), ("Q", C.c_int), ("N", C.c_int), ("c", C.c_int), ("nb", C.c_int),
        ("batch_first", C.POINTER(C.c_int)), ("node_batch", C.POINTER(C.c_int)),
        ("n_packet", C.c_int64),
        ("pkt_recv", C.POINTER(C.c_int)), ("pkt_batch", C.POINTER(C.c_int)), ("pkt_send", C.POINTER(C.c_int)),
    ]


class CompressionPlan:
    """Placement and packet list of the compression-only comparison scheme (appendix)."""

    def __init__(self, K, r, Q, N):
        lib = _load()
        lib.orc_cplan_build.restype = C.POINTER(_CCPlan)
        lib.orc_cplan_build.argtypes = [C.c_int] * 4
        lib.orc_cplan_free.restype = None
        lib.orc_cplan_free.argtypes = [C.POINTER(_CCPlan)]
        lib.orc_cplan_scheduled_elems.restype = C.c_int64
        lib.orc_cplan_scheduled_elems.argtypes = [C.POINTER(_CCPlan), C.c_int64]
        for sfx in ("f64", "u32"):
            for name, nptr in (("ccombine", 2), ("creduce", 3)):
                fn = getattr(lib, f"orc_{name}_{sfx}")
                fn.restype = None
                fn.argtypes = [C.POINTER(_CCPlan), C.c_int64] + [C.c_void_p] * nptr
        ptr = lib.orc_cplan_build(K, r, Q, N)
        if not ptr:
            raise ValueError(f"invalid parameters K={K} r={r} Q={Q} N={N}")
        self._ptr, self._lib = ptr, lib
        s = ptr.contents
        self.K, self.r, self.Q, self.N, self.c, self.nb = s.K, s.r, s.Q, s.N, s.c, s.nb
        self.n_packet = int(s.n_packet)
        self.batch_first = _arr(s.batch_first, (self.nb + 1,))
        self.node_batch = _arr(s.node_batch, (self.K,))
        self.pkt_recv = _arr(s.pkt_recv, (self.n_packet,))
        self.pkt_batch = _arr(s.pkt_batch, (self.n_packet,))
        self.pkt_send = _arr(s.pkt_send, (self.n_packet,))

    def __del__(self):
        try:
            if self._ptr:
                self._lib.orc_cplan_free(self._ptr)
                self._ptr = None
        except Exception:
            pass

    def scheduled_elems(self, T):
        return int(self._lib.orc_cplan_scheduled_elems(self._ptr, T))

    def combine(self, T, V):
        sfx, el = _mode(V)
        _check(V, np.float32 if sfx == "f64" else np.uint32, (self.N, self.Q, T), "V")
        out = np.empty((self.n_packet, self.c * T), dtype=el)
        getattr(self._lib, f"orc_ccombine_{sfx}")(self._ptr, T, _ptr(V), _ptr(out))
        return out

    def reduce(self, T, V, P):
        sfx, el = _mode(V)
        _check(V, np.float32 if sfx == "f64" else np.uint32, (self.N, self.Q, T), "V")
        _check(P, el, (self.n_packet, self.c * T), "P")
        out = np.empty((self.Q, T), dtype=el)
        getattr(self._lib, f"orc_creduce_{sfx}")(self._ptr, T, _ptr(V), _ptr(P), _ptr(out))
        return out


def combine_h32(plan, T, V):
    sh = plan.shapes(T)
    _check(V, np.float32, sh["V"], "V")
    out = np.empty(sh["Vbar"], dtype=np.float32)
    _load().orc_combine_h32(plan._ptr, T, _ptr(V), _ptr(out))
    return out


def encode_h32(plan, T, Vbar):
    sh = plan.shapes(T)
    _check(Vbar, np.float32, sh["Vbar"], "Vbar")
    out = np.empty(sh["X"], dtype=np.uint32)
    _load().orc_encode_h32(plan._ptr, T, _ptr(Vbar), _ptr(out))
    return out


def decode_h32(plan, T, X, Vbar):
    sh = plan.shapes(T)
    _check(X, np.uint32, sh["X"], "X")
    _check(Vbar, np.float32, sh["Vbar"], "Vbar")
    out = np.zeros(sh["D"], dtype=np.float32)
    _load().orc_decode_h32(plan._ptr, T, _ptr(X), _ptr(Vbar), _ptr(out))
    return out


def run_all_h32(plan, T, V):
    """The "h32" algebra: fp32 sums when pre-combining, XOR of bit patterns to code
    and decode, fp64 final reduction.  Vbar/D float32, X uint32, Phi float64."""
    lib = _load()
    sh = plan.shapes(T)
    _check(V, np.float32, sh["V"], "V")
    Vbar = np.empty(sh["Vbar"], dtype=np.float32)
    X = np.empty(sh["X"], dtype=np.uint32)
    D = np.zeros(sh["D"], dtype=np.float32)
    Phi = np.empty(sh["Phi"], dtype=np.float64)
    lib.orc_combine_h32(plan._ptr, T, _ptr(V), _ptr(Vbar))
    lib.orc_encode_h32(plan._ptr, T, _ptr(Vbar), _ptr(X))
    lib.orc_decode_h32(plan._ptr, T, _ptr(X), _ptr(Vbar), _ptr(D))
    lib.orc_reduce_h32(plan._ptr, T, _ptr(V), _ptr(D), _ptr(Phi))
    return {"Vbar": Vbar, "X": X, "D": D, "Phi": Phi}


def run_all(plan, T, V):
    """All four stages in order; returns every artefact."""
    Vbar = combine(plan, T, V)
    X = encode(plan, T, Vbar)
    D = decode(plan, T, X, Vbar)
    Phi = reduce(plan, T, V, D)
    return {"Vbar": Vbar, "X": X, "D": D, "Phi": Phi}


H16_FORMATS = {"bf16": 0, "f16": 1}


def h16_widen(bits, fmt):
    """Exact float32 values of 16-bit patterns (fmt "bf16" or "f16")."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    lib = _load()
    lib.orc_h16_widen(_ptr(bits), _ptr(out), C.c_int64(bits.size), H16_FORMATS[fmt])
    return out


def h16_narrow(values, fmt):
    """Nearest 16-bit patterns (ties to even) of float32 values."""
    values = np.ascontiguousarray(values, dtype=np.float32)
    out = np.empty(values.shape, dtype=np.uint16)
    lib = _load()
    lib.orc_h16_narrow(_ptr(values), _ptr(out), C.c_int64(values.size), H16_FORMATS[fmt])
    return out


def run_all_h16(plan, T, V, fmt):
    """The "h16" algebra on 16-bit patterns V (uint16): Vbar/X/D uint16, Phi float64 (not rounded)."""
    lib = _load()
    f = H16_FORMATS[fmt]
    sh = plan.shapes(T)
    _check(V, np.uint16, sh["V"], "V")
    Vbar = np.empty(sh["Vbar"], dtype=np.uint16)
    X = np.empty(sh["X"], dtype=np.uint16)
    D = np.zeros(sh["D"], dtype=np.uint16)
    Phi = np.empty(sh["Phi"], dtype=np.float64)
    T64 = C.c_int64(T)
    lib.orc_combine_h16(plan._ptr, T64, f, _ptr(V), _ptr(Vbar))
    lib.orc_encode_h16(plan._ptr, T64, _ptr(Vbar), _ptr(X))
    lib.orc_decode_h16(plan._ptr, T64, _ptr(X), _ptr(Vbar), _ptr(D))
    lib.orc_reduce_h16(plan._ptr, T64, f, _ptr(V), _ptr(D), _ptr(Phi))
    return {"Vbar": Vbar, "X": X, "D": D, "Phi": Phi}


def shuffle_h16(plan, T, V, fmt):
    """The three shuffle stages of the "h16" algebra without the final reduction:
    Vbar, X, D as uint16 patterns."""
    lib = _load()
    f = H16_FORMATS[fmt]
    sh = plan.shapes(T)
    _check(V, np.uint16, sh["V"], "V")
    Vbar = np.empty(sh["Vbar"], dtype=np.uint16)
    X = np.empty(sh["X"], dtype=np.uint16)
    D = np.zeros(sh["D"], dtype=np.uint16)
    T64 = C.c_int64(T)
    lib.orc_combine_h16(plan._ptr, T64, f, _ptr(V), _ptr(Vbar))
    lib.orc_encode_h16(plan._ptr, T64, _ptr(Vbar), _ptr(X))
    lib.orc_decode_h16(plan._ptr, T64, _ptr(X), _ptr(Vbar), _ptr(D))
    return {"Vbar": Vbar, "X": X, "D": D}


def direct_h16(plan, T, V, fmt):
    """eq. (1) on 16-bit inputs, fp64."""
    sh = plan.shapes(T)
    _check(V, np.uint16, sh["V"], "V")
    out = np.empty(sh["Phi"], dtype=np.float64)
    _load().orc_direct_h16(plan._ptr, C.c_int64(T), H16_FORMATS[fmt], _ptr(V), _ptr(out))
    return out


def map_files(files, theta, fmt=None):
    """Map stand-in (Sec. III): V[j][n][q][t] = theta[j][q][t] - files[j][n][q][t].
    float32 arrays: one fp32 subtraction; uint32: XOR; uint16 patterns with fmt "bf16" /
    "f16": the fp32 difference rounded once to the format."""
    lib = _load()
    J, N, Q, T = files.shape
    _check(files, files.dtype, (J, N, Q, T), "files")
    _check(theta, files.dtype, (J, Q, T), "theta")
    out = np.empty_like(files)
    if files.dtype == np.float32:
        lib.orc_map_f32(J, N, Q, C.c_int64(T), _ptr(files), _ptr(theta), _ptr(out))
    elif files.dtype == np.uint32:
        lib.orc_map_u32(J, N, Q, C.c_int64(T), _ptr(files), _ptr(theta), _ptr(out))
    elif files.dtype == np.uint16:
        lib.orc_map_h16(J, N, Q, C.c_int64(T), H16_FORMATS[fmt], _ptr(files), _ptr(theta), _ptr(out))
    else:
        raise TypeError(f"unsupported dtype {files.dtype}")
    return out
