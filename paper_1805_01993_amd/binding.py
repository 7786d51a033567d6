"""ctypes binding of libccdc.so: same names as the C entry points, argument
marshalling only.  PyTorch supplies device memory and streams; every step of
the path runs in the library's kernels.  There is no CPU fallback: a missing
or unloadable library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libccdc.so")

OK, EINVAL, ENOMEM, EHIP, ESIZE, ESTATE = 0, -1, -2, -3, -4, -5
F32_SUM, U32_XOR, F32_SUM_XOR, BF16_SUM_XOR, F16_SUM_XOR = 0, 1, 2, 3, 4
MODES = {"f32": F32_SUM, "u32": U32_XOR, "h32": F32_SUM_XOR, "bf16": BF16_SUM_XOR, "f16": F16_SUM_XOR}
ELEM_BYTES = {F32_SUM: 4, U32_XOR: 4, F32_SUM_XOR: 4, BF16_SUM_XOR: 2, F16_SUM_XOR: 2}

# enum ccdc_query
(Q_K, Q_R, Q_Q, Q_N, Q_J, Q_C, Q_M, Q_NBATCH, Q_NROUND, Q_T, Q_MODE, Q_W, Q_SEG_LEN,
 Q_SCHEDULED_ELEMS, Q_CLOSED_FORM_NUM, Q_CLOSED_FORM_DEN, Q_V_ELEMS, Q_VBAR_ELEMS, Q_X_ELEMS,
 Q_D_ELEMS, Q_PHI_ELEMS, Q_WORKSPACE_BYTES) = range(22)
(Q_PACKET_LEN, Q_BATCH_JOB, Q_BATCH_FILE0, Q_BATCH_LABEL, Q_ROUND_MEMBER, Q_ROUND_BATCH) = range(64, 70)
(Q_NROWS, Q_SCHEME, Q_BATCH_FIRST, Q_NODE_BATCH, Q_PACKET_RECV, Q_PACKET_BATCH, Q_PACKET_SEND,
 Q_ROWS_PER_NODE, Q_NODE_ROWS, Q_FILE_NODES, Q_FILES_PER_NODE, Q_NODE_FILES) = range(128, 140)

EXPORTS = [
    "ccdc_plan", "ccdc_plan_jobs", "ccdc_plan_jobs_repeated", "ccdc_plan_compression", "ccdc_plan_destroy", "ccdc_plan_bind", "ccdc_plan_upload",
    "ccdc_plan_query", "ccdc_strerror", "ccdc_map", "ccdc_combine", "ccdc_encode", "ccdc_decode", "ccdc_reduce",
    "ccdc_shuffle_fused", "ccdc_pipeline_fused", "ccdc_pipeline_fused_noalloc", "ccdc_node_encode",
    "ccdc_node_decode_reduce",
]


class CcdcError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def load_library():
    """Load libccdc.so (built in-tree by build.py).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it first (python -m paper_1805_01993_amd.build "
            "or __graft_entry__.build()); there is no fallback path")
    try:
        import torch  # noqa: F401  (loads the HIP runtime the process will share)
    except Exception:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i64 = C.c_void_p, C.c_int64
    lib.ccdc_plan.restype = C.c_int
    lib.ccdc_plan.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    lib.ccdc_plan_jobs.restype = C.c_int
    lib.ccdc_plan_jobs.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    lib.ccdc_plan_jobs_repeated.restype = C.c_int
    lib.ccdc_plan_jobs_repeated.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    lib.ccdc_plan_compression.restype = C.c_int
    lib.ccdc_plan_compression.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(vp)]
    lib.ccdc_plan_destroy.restype = None
    lib.ccdc_plan_destroy.argtypes = [vp]
    lib.ccdc_plan_bind.restype = C.c_int
    lib.ccdc_plan_bind.argtypes = [vp, i64, C.c_int]
    lib.ccdc_plan_upload.restype = C.c_int
    lib.ccdc_plan_upload.argtypes = [vp]
    lib.ccdc_plan_query.restype = C.c_int
    lib.ccdc_plan_query.argtypes = [vp, C.c_int, vp, C.c_size_t]
    lib.ccdc_strerror.restype = C.c_char_p
    lib.ccdc_strerror.argtypes = [C.c_int]
    for name, nptr in (("ccdc_combine", 2), ("ccdc_encode", 2), ("ccdc_decode", 3), ("ccdc_reduce", 3),
                       ("ccdc_shuffle_fused", 3), ("ccdc_pipeline_fused", 3), ("ccdc_pipeline_fused_noalloc", 3),
                       ("ccdc_map", 3)):
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = [vp] + [vp] * nptr + [vp]
    for name, nptr in (("ccdc_node_encode", 2), ("ccdc_node_decode_reduce", 3)):
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = [vp, C.c_int] + [vp] * nptr + [vp]
    _lib = lib
    return lib


def strerror(status):
    return load_library().ccdc_strerror(status).decode()


def _check(status, where):
    if status != OK:
        raise CcdcError(status, where)


def _dev_ptr(t, name, elem_bytes=4):
    """Device address of a contiguous CUDA/HIP torch tensor."""
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name}: need a contiguous device tensor")
    if t.element_size() != elem_bytes:
        raise ValueError(f"{name}: need {elem_bytes}-byte elements, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


class Plan:
    """Owns one ccdc_plan_t.  Methods mirror the C entry points."""

    def __init__(self, K, r, Q, N, jobs=False, compression=False, gamma=1):
        lib = load_library()
        h = C.c_void_p()
        if gamma != 1:
            if not jobs:
                raise ValueError("gamma repeats the J-job schedule: pass jobs=True")
            _check(lib.ccdc_plan_jobs_repeated(K, r, Q, N, int(gamma), C.byref(h)), "ccdc_plan_jobs_repeated")
        else:
            name = "ccdc_plan_compression" if compression else ("ccdc_plan_jobs" if jobs else "ccdc_plan")
            _check(getattr(lib, name)(K, r, Q, N, C.byref(h)), name)
        self._h = h
        self.compression = bool(compression)
        self._lib = lib
        self._shapes = None

    def close(self):
        if getattr(self, "_h", None):
            self._lib.ccdc_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- plan construction
    def bind(self, T, mode):
        mode = MODES.get(mode, mode)
        _check(self._lib.ccdc_plan_bind(self._h, int(T), mode), "ccdc_plan_bind")
        self._shapes = None
        self._elem_bytes = ELEM_BYTES[mode]
        return self

    def upload(self):
        _check(self._lib.ccdc_plan_upload(self._h), "ccdc_plan_upload")
        return self

    # ---- introspection
    def query(self, what):
        v = C.c_int64()
        _check(self._lib.ccdc_plan_query(self._h, what, C.byref(v), 8), f"ccdc_plan_query({what})")
        return int(v.value)

    def query_table(self, what, shape, dtype):
        out = np.empty(shape, dtype=dtype)
        _check(self._lib.ccdc_plan_query(self._h, what, out.ctypes.data_as(C.c_void_p), out.nbytes),
               f"ccdc_plan_query({what})")
        return out

    @property
    def K(self): return self.query(Q_K)
    @property
    def r(self): return self.query(Q_R)
    @property
    def Q(self): return self.query(Q_Q)
    @property
    def N(self): return self.query(Q_N)
    @property
    def J(self): return self.query(Q_J)
    @property
    def c(self): return self.query(Q_C)
    @property
    def m(self): return self.query(Q_M)
    @property
    def n_batch(self): return self.query(Q_NBATCH)
    @property
    def n_round(self): return self.query(Q_NROUND)
    @property
    def T(self): return self.query(Q_T)
    @property
    def W(self): return self.query(Q_W)
    @property
    def seg_len(self): return self.query(Q_SEG_LEN)
    @property
    def scheduled_elems(self): return self.query(Q_SCHEDULED_ELEMS)
    @property
    def closed_form_elems(self):
        return Fraction(self.query(Q_CLOSED_FORM_NUM), self.query(Q_CLOSED_FORM_DEN))
    @property
    def workspace_bytes(self): return self.query(Q_WORKSPACE_BYTES)

    def tables(self):
        nb, R, r = self.n_batch, self.n_round, self.r
        return {
            "batch_job": self.query_table(Q_BATCH_JOB, (nb,), np.int32),
            "batch_file0": self.query_table(Q_BATCH_FILE0, (nb,), np.int32),
            "batch_label": self.query_table(Q_BATCH_LABEL, (nb, r), np.int32),
            "round_member": self.query_table(Q_ROUND_MEMBER, (R, r + 1), np.int32),
            "round_batch": self.query_table(Q_ROUND_BATCH, (R, r + 1), np.int32),
        }

    def node_rows(self):
        """[K][rows per node]: the packets u*(r+1)+a each node sends (coded plans)."""
        return self.query_table(Q_NODE_ROWS, (self.K, self.query(Q_ROWS_PER_NODE)), np.int32)

    def file_nodes(self):
        """[J*N][r]: the r nodes that store file job*N + n (placement of Sec. IV-A)."""
        return self.query_table(Q_FILE_NODES, (self.J * self.N, self.r), np.int32)

    def node_files(self):
        """[K][files per node]: the set M_k of files each node stores, ascending."""
        return self.query_table(Q_NODE_FILES, (self.K, self.query(Q_FILES_PER_NODE)), np.int32)

    def packet_len(self):
        return self.query_table(Q_PACKET_LEN, (1 if self.compression else self.r + 1,), np.int64)

    def compression_tables(self):
        nb, rows = self.n_batch, self.query(Q_NROWS)
        return {
            "batch_first": self.query_table(Q_BATCH_FIRST, (nb + 1,), np.int32),
            "node_batch": self.query_table(Q_NODE_BATCH, (self.K,), np.int32),
            "pkt_recv": self.query_table(Q_PACKET_RECV, (rows,), np.int32),
            "pkt_batch": self.query_table(Q_PACKET_BATCH, (rows,), np.int32),
            "pkt_send": self.query_table(Q_PACKET_SEND, (rows,), np.int32),
        }

    def shapes(self):
        if self._shapes is None:          # fixed by bind(); queried once
            R, r1, W, ell = self.n_round, self.r + 1, self.W, self.seg_len
            if self.compression:          # uncoded packets only: K receivers x (nb-1) batches
                rows = self.query(Q_NROWS)
                self._shapes = {"V": (1, self.N, self.Q, self.T), "Vbar": (rows, W), "X": (0,),
                                "D": (rows, W), "Phi": (1, self.Q, self.T)}
            else:
                self._shapes = {"V": (self.J, self.N, self.Q, self.T), "Vbar": (R, r1, W), "X": (R, r1, ell),
                                "D": (R, r1, W), "Phi": (self.J, self.Q, self.T)}
            self._numel = {k: int(np.prod(v)) for k, v in self._shapes.items()}
        return self._shapes

    def _need(self, t, key, name):
        self.shapes()
        want = self._numel[key]
        if t.numel() != want:
            raise ValueError(f"{name}: need {want} elements, got {t.numel()}")
        return _dev_ptr(t, name, self._elem_bytes)

    # ---- Map stand-in: V = theta - files (V may be the files tensor itself)
    def map(self, files, theta, V, stream=None):
        _check(self._lib.ccdc_map(self._h, self._need(files, "V", "files"), self._need(theta, "Phi", "theta"),
                                  self._need(V, "V", "V"), _stream_ptr(stream)), "ccdc_map")

    # ---- stages (asynchronous on `stream`, default torch's current stream)
    def combine(self, V, Vbar, stream=None):
        _check(self._lib.ccdc_combine(self._h, self._need(V, "V", "V"), self._need(Vbar, "Vbar", "Vbar"),
                                      _stream_ptr(stream)), "ccdc_combine")

    def encode(self, Vbar, X, stream=None):
        _check(self._lib.ccdc_encode(self._h, self._need(Vbar, "Vbar", "Vbar"), self._need(X, "X", "X"),
                                     _stream_ptr(stream)), "ccdc_encode")

    def decode(self, X, Vbar, D, stream=None):
        _check(self._lib.ccdc_decode(self._h, self._need(X, "X", "X"), self._need(Vbar, "Vbar", "Vbar"),
                                     self._need(D, "D", "D"), _stream_ptr(stream)), "ccdc_decode")

    def reduce(self, V, D, Phi, stream=None):
        _check(self._lib.ccdc_reduce(self._h, self._need(V, "V", "V"), self._need(D, "D", "D"),
                                     self._need(Phi, "Phi", "Phi"), _stream_ptr(stream)), "ccdc_reduce")

    def shuffle_fused(self, V, X, D, stream=None):
        _check(self._lib.ccdc_shuffle_fused(self._h, self._need(V, "V", "V"), self._need(X, "X", "X"),
                                            self._need(D, "D", "D"), _stream_ptr(stream)), "ccdc_shuffle_fused")

    def pipeline_fused(self, V, X, Phi, stream=None):
        _check(self._lib.ccdc_pipeline_fused(self._h, self._need(V, "V", "V"), self._need(X, "X", "X"),
                                             self._need(Phi, "Phi", "Phi"), _stream_ptr(stream)),
               "ccdc_pipeline_fused")

    def pipeline_fused_noalloc(self, V, X, Phi, stream=None):
        _check(self._lib.ccdc_pipeline_fused_noalloc(self._h, self._need(V, "V", "V"), self._need(X, "X", "X"),
                                                     self._need(Phi, "Phi", "Phi"), _stream_ptr(stream)),
               "ccdc_pipeline_fused_noalloc")

    # ---- the node-local form: node = -1 runs every node
    def node_encode(self, node, V, X, stream=None):
        _check(self._lib.ccdc_node_encode(self._h, int(node), self._need(V, "V", "V"), self._need(X, "X", "X"),
                                          _stream_ptr(stream)), "ccdc_node_encode")

    def node_decode_reduce(self, node, V, X, Phi, stream=None):
        _check(self._lib.ccdc_node_decode_reduce(self._h, int(node), self._need(V, "V", "V"), self._need(X, "X", "X"),
                                                 self._need(Phi, "Phi", "Phi"), _stream_ptr(stream)),
               "ccdc_node_decode_reduce")


def ccdc_plan(K, r, Q, N):
    """Single-job placement and schedule (one batch per r-subset of the cluster)."""
    return Plan(K, r, Q, N, jobs=False)


def ccdc_plan_jobs(K, r, Q, N):
    """The paper's J = C(K, r+1)-job placement and two-stage schedule."""
    return Plan(K, r, Q, N, jobs=True)


def ccdc_plan_jobs_repeated(K, r, Q, N, gamma):
    """The J-job scheme repeated on gamma consecutive blocks of C(K, r+1) jobs."""
    return Plan(K, r, Q, N, jobs=True, gamma=gamma)


def ccdc_plan_compression(K, r, Q, N):
    """The compression-only comparison scheme (appendix): cyclic batches, uncoded packets."""
    return Plan(K, r, Q, N, compression=True)
