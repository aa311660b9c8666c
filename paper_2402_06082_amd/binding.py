"""Thin ctypes binding of libsubgen.so (``include/subgen.h``), same names as the C ABI.

Argument marshalling only: every step of the decode path runs in the HIP
kernels of the library.  PyTorch appears here as the owner of device buffers
and of the HIP stream.  There is no fallback: if the library has not been
built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional

import numpy as np
import torch

_LIB_PATH = Path(__file__).resolve().parent / "libsubgen.so"
_lib = None

SUBGEN_F32, SUBGEN_BF16 = 0, 1
FLAG_CENTER_OVERFLOW = 1
FLAG_NONFINITE = 2

EXPORTS = [
    "subgen_create", "subgen_destroy", "subgen_update", "subgen_attend", "subgen_attend_many", "subgen_step",
    "subgen_ingest_prefix",
    "subgen_exact_workspace_bytes", "subgen_exact_attend", "subgen_exact_noalloc_max_bytes",
    "subgen_exact_attend_noalloc", "subgen_hbm_read_probe", "subgen_kcenter_workspace_bytes",
    "subgen_kcenter_compress", "subgen_stats", "subgen_center_counts",
    "subgen_export_state", "subgen_import_state", "subgen_sync", "subgen_strerror", "subgen_last_hip_error",
]


class SubgenError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


class subgen_opts(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("dtype", C.c_int32), ("q_per_stream", C.c_int32),
                ("max_centers", C.c_int32), ("assign_log_tokens", C.c_int64), ("seed", C.c_uint64),
                ("hip_stream", C.c_void_p), ("device", C.c_int32), ("device_set", C.c_int32),
                ("kernel_path", C.c_int32), ("t_per_cluster", C.c_int32), ("device_counter", C.c_int32),
                ("out_dtype", C.c_int32), ("split_workgroups", C.c_int32), ("reserved_", C.c_int32)]


class subgen_stats_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("flags_or", C.c_uint32), ("streams", C.c_int64),
                ("n_seen", C.c_int64), ("n_evicted", C.c_int64), ("total_centers", C.c_int64),
                ("min_centers", C.c_int32), ("max_centers", C.c_int32), ("flagged_streams", C.c_int64)]


class subgen_state_view(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("flags", C.c_uint32), ("m", C.c_int32), ("window_fill", C.c_int32),
                ("n_seen", C.c_int64), ("n_evicted", C.c_int64), ("mu", C.c_double),
                ("centers_cap", C.c_int64), ("centers", C.c_void_p), ("counts", C.c_void_p),
                ("sample_K", C.c_void_p), ("sample_V", C.c_void_p), ("sample_idx", C.c_void_p),
                ("sample_vn", C.c_void_p), ("window_K", C.c_void_p), ("window_V", C.c_void_p),
                ("assign_cap", C.c_int64), ("assign", C.c_void_p), ("assign_len", C.c_int64),
                ("reservoirs", C.c_void_p)]


def lib_path() -> Path:
    return _LIB_PATH


def load():
    """Load libsubgen.so; raises if it has not been built (there is no other path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not _LIB_PATH.exists():
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2402_06082_amd.build` "
                           "(the decode path has no CPU fallback)")
    L = C.CDLL(str(_LIB_PATH))
    P, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.subgen_create.restype = C.c_int
    L.subgen_create.argtypes = [C.POINTER(P), i64, i32, C.c_float, i32, i32, C.POINTER(subgen_opts)]
    L.subgen_destroy.restype = None
    L.subgen_destroy.argtypes = [P]
    L.subgen_update.restype = C.c_int
    L.subgen_update.argtypes = [P, P, P]
    L.subgen_attend.restype = C.c_int
    L.subgen_attend.argtypes = [P, P, P]
    L.subgen_attend_many.restype = C.c_int
    L.subgen_attend_many.argtypes = [P, P, i32, P]
    L.subgen_step.restype = C.c_int
    L.subgen_step.argtypes = [P, P, P, P, P]
    L.subgen_ingest_prefix.restype = C.c_int
    L.subgen_ingest_prefix.argtypes = [P, P, P, i64, i64, i64]
    L.subgen_exact_workspace_bytes.restype = C.c_size_t
    L.subgen_exact_workspace_bytes.argtypes = [i64, i64, i32, i32]
    L.subgen_exact_attend.restype = C.c_int
    L.subgen_exact_attend.argtypes = [P, P, P, P, i64, i64, i32, i32, i32, P, C.c_size_t, P]
    L.subgen_exact_noalloc_max_bytes.restype = C.c_size_t
    L.subgen_exact_noalloc_max_bytes.argtypes = []
    L.subgen_exact_attend_noalloc.restype = C.c_int
    L.subgen_exact_attend_noalloc.argtypes = [P, P, P, P, i64, i64, i32, i32, i32, P]
    L.subgen_kcenter_workspace_bytes.restype = C.c_size_t
    L.subgen_kcenter_workspace_bytes.argtypes = [i64, i64, i32]
    L.subgen_kcenter_compress.restype = C.c_int
    L.subgen_kcenter_compress.argtypes = [P, P, i64, i64, i32, i32, i32, i32, P, P, P, P, P, C.c_size_t, P]
    L.subgen_hbm_read_probe.restype = C.c_int
    L.subgen_hbm_read_probe.argtypes = [P, C.c_size_t, i32, i32, C.c_size_t, P, P]
    L.subgen_stats.restype = C.c_int
    L.subgen_stats.argtypes = [P, C.POINTER(subgen_stats_t)]
    L.subgen_center_counts.restype = C.c_int
    L.subgen_center_counts.argtypes = [P, P]
    L.subgen_export_state.restype = C.c_int
    L.subgen_export_state.argtypes = [P, i64, C.POINTER(subgen_state_view)]
    L.subgen_import_state.restype = C.c_int
    L.subgen_import_state.argtypes = [P, i64, C.POINTER(subgen_state_view)]
    L.subgen_sync.restype = C.c_int
    L.subgen_sync.argtypes = [P]
    L.subgen_strerror.restype = C.c_char_p
    L.subgen_strerror.argtypes = [C.c_int]
    L.subgen_last_hip_error.restype = C.c_int
    L.subgen_last_hip_error.argtypes = [P]
    _lib = L
    return L


def strerror(code: int) -> str:
    return load().subgen_strerror(int(code)).decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise SubgenError(rc, what)


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return SUBGEN_F32
    if dt == torch.bfloat16:
        return SUBGEN_BF16
    raise ValueError(f"unsupported dtype {dt}")


def _np_rows(dtype_code: int, rows: int, d: int) -> np.ndarray:
    return np.zeros((rows, d), dtype=np.float32 if dtype_code == SUBGEN_F32 else np.uint16)


def _rows_to_f32(a: np.ndarray) -> np.ndarray:
    """Host rows (fp32, or bf16 bit patterns as uint16) -> float32 values."""
    if a.dtype == np.float32:
        return a
    return (a.astype(np.uint32) << 16).view(np.float32)


class StreamState:
    """Host copy of one stream's state (rows converted to float32 values)."""
    __slots__ = ("m", "n_seen", "n_evicted", "mu", "flags", "window_fill", "centers", "counts", "sample_k",
                 "sample_v", "sample_idx", "sample_vn", "window_k", "window_v", "assign", "reservoirs")


class SubGen:
    """One context: ``streams`` independent SubGen streams advancing in lock-step."""

    def __init__(self, streams: int, d: int, delta: float, sample_budget: int, window: int, *,
                 dtype: torch.dtype = torch.float32, q_per_stream: int = 1, max_centers: int = 0,
                 assign_log_tokens: int = 0, seed: int = 0, device: Optional[torch.device] = None,
                 kernel_path: int = 0, t_per_cluster: int = 0, device_counter: bool = False,
                 out_dtype: torch.dtype = torch.float32, split_workgroups: int = 0):
        self._L = load()
        self._h = C.c_void_p()
        if not torch.cuda.is_available():
            raise RuntimeError("SubGen needs a GPU: the decode path has no CPU fallback")
        self.device = torch.device(device if device is not None else "cuda:0")
        self.streams, self.d, self.s, self.w = int(streams), int(d), int(sample_budget), int(window)
        self.g = int(q_per_stream)
        self.dtype = dtype
        self.dtype_code = _dtype_code(dtype)
        self.out_dtype = out_dtype
        self.max_centers = int(max_centers) if max_centers else 4096
        self.assign_log_tokens = int(assign_log_tokens)
        self.delta = float(np.float32(delta))
        o = subgen_opts()
        o.struct_size = C.sizeof(subgen_opts)
        o.dtype = self.dtype_code
        o.q_per_stream = self.g
        o.max_centers = int(max_centers)
        o.assign_log_tokens = self.assign_log_tokens
        o.seed = int(seed)
        o.hip_stream = torch.cuda.current_stream(self.device).cuda_stream
        o.device = self.device.index or 0
        o.device_set = 1
        o.kernel_path = int(kernel_path)
        o.device_counter = 1 if device_counter else 0
        o.t_per_cluster = self.t = int(t_per_cluster)
        o.out_dtype = _dtype_code(out_dtype)
        o.split_workgroups = int(split_workgroups)
        _check(self._L.subgen_create(C.byref(self._h), self.streams, self.d, C.c_float(self.delta), self.s, self.w,
                                     C.byref(o)), "subgen_create")

    def close(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            self._L.subgen_destroy(h)

    def __del__(self):
        self.close()

    # -- argument checks (shape / dtype / device / contiguity) ---------------
    def _rows(self, t: torch.Tensor, shape, what: str, dtype=None):
        if tuple(t.shape) != tuple(shape) or t.dtype != (dtype or self.dtype) or not t.is_cuda \
                or not t.is_contiguous():
            raise ValueError(f"{what}: expected contiguous {dtype or self.dtype} cuda tensor of shape {tuple(shape)}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}")
        return C.c_void_p(t.data_ptr())

    # -- the C entry points ---------------------------------------------------
    def update(self, K_t: torch.Tensor, V_t: torch.Tensor) -> None:
        k = self._rows(K_t, (self.streams, self.d), "K_t")
        v = self._rows(V_t, (self.streams, self.d), "V_t")
        _check(self._L.subgen_update(self._h, k, v), "subgen_update")

    def attend(self, Q_t: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        if out is None:
            out = torch.empty(self.streams, self.g, self.d, dtype=self.out_dtype, device=self.device)
        q = self._rows(Q_t, (self.streams, self.g, self.d), "Q_t")
        o = self._rows(out, (self.streams, self.g, self.d), "out", self.out_dtype)
        _check(self._L.subgen_attend(self._h, q, o), "subgen_attend")
        return out

    def attend_many(self, Q: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Q [streams, n_queries, d] -> out [streams, n_queries, d] fp32; every query as in ``attend``."""
        if Q.dim() != 3:
            raise ValueError("Q must be [streams, n_queries, d]")
        nq = int(Q.shape[1])
        if out is None:
            out = torch.empty(self.streams, nq, self.d, dtype=self.out_dtype, device=self.device)
        q = self._rows(Q, (self.streams, nq, self.d), "Q")
        o = self._rows(out, (self.streams, nq, self.d), "out", self.out_dtype)
        _check(self._L.subgen_attend_many(self._h, q, nq, o), "subgen_attend_many")
        return out

    def step(self, K_t: torch.Tensor, V_t: torch.Tensor, Q_t: torch.Tensor,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
        if out is None:
            out = torch.empty(self.streams, self.g, self.d, dtype=self.out_dtype, device=self.device)
        k = self._rows(K_t, (self.streams, self.d), "K_t")
        v = self._rows(V_t, (self.streams, self.d), "V_t")
        q = self._rows(Q_t, (self.streams, self.g, self.d), "Q_t")
        o = self._rows(out, (self.streams, self.g, self.d), "out", self.out_dtype)
        _check(self._L.subgen_step(self._h, k, v, q, o), "subgen_step")
        return out

    def ingest_prefix(self, K: torch.Tensor, V: torch.Tensor) -> None:
        """K, V: [streams, n, d]; any strides with a unit last stride."""
        for t, what in ((K, "K"), (V, "V")):
            if t.dim() != 3 or t.shape[0] != self.streams or t.shape[2] != self.d or t.dtype != self.dtype \
                    or not t.is_cuda or (t.shape[1] > 0 and t.stride(2) != 1):
                raise ValueError(f"{what}: expected [streams, n, d] {self.dtype} cuda tensor")
        if K.shape != V.shape or K.stride() != V.stride():
            raise ValueError("K and V must have the same shape and strides")
        n = K.shape[1]
        _check(self._L.subgen_ingest_prefix(self._h, C.c_void_p(K.data_ptr()), C.c_void_p(V.data_ptr()), n,
                                            K.stride(0), K.stride(1)), "subgen_ingest_prefix")

    def sync(self) -> None:
        _check(self._L.subgen_sync(self._h), "subgen_sync")

    def stats(self) -> subgen_stats_t:
        st = subgen_stats_t()
        _check(self._L.subgen_stats(self._h, C.byref(st)), "subgen_stats")
        return st

    def center_counts(self) -> np.ndarray:
        m = np.zeros(self.streams, dtype=np.int32)
        _check(self._L.subgen_center_counts(self._h, m.ctypes.data_as(C.c_void_p)), "subgen_center_counts")
        return m

    def export_raw(self, stream: int) -> dict:
        """One stream's state as host arrays in the library's own element format (for import_raw)."""
        v = subgen_state_view()
        v.struct_size = C.sizeof(subgen_state_view)
        cap = self.max_centers
        bufs = {
            "centers": _np_rows(self.dtype_code, cap, self.d), "counts": np.zeros(cap, dtype=np.int32),
            "sample_K": _np_rows(self.dtype_code, self.s, self.d), "sample_V": _np_rows(self.dtype_code, self.s, self.d),
            "sample_idx": np.zeros(self.s, dtype=np.int32), "sample_vn": np.zeros(self.s, dtype=np.float32),
            "window_K": _np_rows(self.dtype_code, max(self.w, 1), self.d),
            "window_V": _np_rows(self.dtype_code, max(self.w, 1), self.d),
        }
        if self.t > 0:
            bufs["reservoirs"] = _np_rows(self.dtype_code, cap * self.t, self.d)
        v.centers_cap = cap
        for k, a in bufs.items():
            setattr(v, k, a.ctypes.data)
        _check(self._L.subgen_export_state(self._h, int(stream), C.byref(v)), "subgen_export_state")
        bufs.update(m=v.m, n_seen=v.n_seen, mu=v.mu, flags=v.flags)
        return bufs

    def import_raw(self, stream: int, state: dict) -> None:
        """Load a stream's state produced by export_raw (possibly of another context with the same shape)."""
        v = subgen_state_view()
        v.struct_size = C.sizeof(subgen_state_view)
        v.m, v.n_seen, v.mu, v.flags = state["m"], state["n_seen"], state["mu"], state["flags"]
        v.centers_cap = state["centers"].shape[0]
        for k in ("centers", "counts", "sample_K", "sample_V", "sample_idx", "sample_vn", "window_K", "window_V",
                  "reservoirs"):
            if k in state:
                setattr(v, k, np.ascontiguousarray(state[k]).ctypes.data)
        _check(self._L.subgen_import_state(self._h, int(stream), C.byref(v)), "subgen_import_state")

    def export_state(self, stream: int, rows: bool = True) -> StreamState:
        v = subgen_state_view()
        v.struct_size = C.sizeof(subgen_state_view)
        cap = self.max_centers
        counts = np.zeros(cap, dtype=np.int32)
        sidx = np.zeros(self.s, dtype=np.int32)
        svn = np.zeros(self.s, dtype=np.float32)
        v.centers_cap = cap
        v.counts = counts.ctypes.data
        v.sample_idx = sidx.ctypes.data
        v.sample_vn = svn.ctypes.data
        if rows:
            centers = _np_rows(self.dtype_code, cap, self.d)
            sk, sv = _np_rows(self.dtype_code, self.s, self.d), _np_rows(self.dtype_code, self.s, self.d)
            wk, wv = _np_rows(self.dtype_code, self.w, self.d), _np_rows(self.dtype_code, self.w, self.d)
            v.centers, v.sample_K, v.sample_V = centers.ctypes.data, sk.ctypes.data, sv.ctypes.data
            v.window_K, v.window_V = wk.ctypes.data, wv.ctypes.data
        res = None
        if rows and self.t > 0:
            res = _np_rows(self.dtype_code, cap * self.t, self.d)
            v.reservoirs = res.ctypes.data
        assign = None
        if self.assign_log_tokens > 0:
            assign = np.zeros(self.assign_log_tokens, dtype=np.int32)
            v.assign, v.assign_cap = assign.ctypes.data, self.assign_log_tokens
        _check(self._L.subgen_export_state(self._h, int(stream), C.byref(v)), "subgen_export_state")
        st = StreamState()
        st.m, st.n_seen, st.n_evicted, st.mu, st.flags = v.m, v.n_seen, v.n_evicted, v.mu, v.flags
        st.window_fill = v.window_fill
        st.counts = counts[: v.m].copy()
        st.sample_idx, st.sample_vn = sidx, svn
        st.assign = assign[: v.assign_len].copy() if assign is not None else None
        if rows:
            st.centers = _rows_to_f32(centers[: v.m])
            st.sample_k, st.sample_v = _rows_to_f32(sk), _rows_to_f32(sv)
            st.window_k, st.window_v = _rows_to_f32(wk)[: v.window_fill], _rows_to_f32(wv)[: v.window_fill]
            st.reservoirs = (_rows_to_f32(res)[: v.m * self.t].reshape(v.m, self.t, self.d)
                             if res is not None else None)
        else:
            st.reservoirs = None
            st.centers = st.sample_k = st.sample_v = st.window_k = st.window_v = None
        return st


def exact_attend(K: torch.Tensor, V: torch.Tensor, Q: torch.Tensor, out: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Exact full-KV decode attention: K, V [streams, n, d], Q [streams, g, d] -> [streams, g, d] fp32."""
    L = load()
    S, n, d = K.shape
    g = Q.shape[1]
    for t in (K, V, Q):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != K.dtype:
            raise ValueError("exact_attend: contiguous cuda tensors of one dtype expected")
    if V.shape != K.shape or tuple(Q.shape) != (S, g, d):
        raise ValueError("exact_attend: shape mismatch")
    if out is None:
        out = torch.empty(S, g, d, dtype=torch.float32, device=K.device)
    need = L.subgen_exact_workspace_bytes(S, n, d, g)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=K.device)
    _check(L.subgen_exact_attend(C.c_void_p(K.data_ptr()), C.c_void_p(V.data_ptr()), C.c_void_p(Q.data_ptr()),
                                 C.c_void_p(out.data_ptr()), S, n, d, g, _dtype_code(K.dtype),
                                 C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                 C.c_void_p(torch.cuda.current_stream(K.device).cuda_stream)), "subgen_exact_attend")
    return out


def exact_attend_noalloc(K: torch.Tensor, V: torch.Tensor, Q: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """subgen_exact_attend_noalloc: as exact_attend, the caller brings ``out`` and nothing is allocated."""
    L = load()
    S, n, d = K.shape
    g = Q.shape[1]
    for t in (K, V, Q):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != K.dtype:
            raise ValueError("exact_attend_noalloc: contiguous cuda tensors of one dtype expected")
    if V.shape != K.shape or tuple(Q.shape) != (S, g, d) or tuple(out.shape) != (S, g, d) \
            or out.dtype != torch.float32 or not out.is_cuda or not out.is_contiguous():
        raise ValueError("exact_attend_noalloc: shape mismatch")
    _check(L.subgen_exact_attend_noalloc(C.c_void_p(K.data_ptr()), C.c_void_p(V.data_ptr()),
                                         C.c_void_p(Q.data_ptr()), C.c_void_p(out.data_ptr()), S, n, d, g,
                                         _dtype_code(K.dtype),
                                         C.c_void_p(torch.cuda.current_stream(K.device).cuda_stream)),
           "subgen_exact_attend_noalloc")
    return out


def hbm_read_probe(buf: torch.Tensor, workgroups: int, sink: torch.Tensor, nontemporal: bool = True,
                   region_bytes: int = 0) -> None:
    """One plain streaming read of ``buf`` (measurement aid; time it with events around the call)."""
    _check(load().subgen_hbm_read_probe(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), int(workgroups),
                                        int(bool(nontemporal)), int(region_bytes), C.c_void_p(sink.data_ptr()),
                                        C.c_void_p(torch.cuda.current_stream(buf.device).cuda_stream)),
           "subgen_hbm_read_probe")


def kcenter_compress(K: torch.Tensor, V: torch.Tensor, k: int, r: int, with_counts: bool = True):
    """Greedy k-center compression of [streams, n, d] caches: returns (K', V', idx, counts) with k + r rows each."""
    L = load()
    S, n, d = K.shape
    for t in (K, V):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != K.dtype or t.shape != K.shape:
            raise ValueError("kcenter_compress: contiguous cuda tensors of one dtype and shape expected")
    oK = torch.empty(S, k + r, d, dtype=K.dtype, device=K.device)
    oV = torch.empty_like(oK)
    idx = torch.empty(S, k + r, dtype=torch.int32, device=K.device)
    counts = torch.empty(S, k, dtype=torch.int32, device=K.device) if with_counts else None
    ws = torch.empty(L.subgen_kcenter_workspace_bytes(S, n, r), dtype=torch.uint8, device=K.device)
    _check(L.subgen_kcenter_compress(C.c_void_p(K.data_ptr()), C.c_void_p(V.data_ptr()), S, n, d, _dtype_code(K.dtype),
                                     int(k), int(r), C.c_void_p(oK.data_ptr()), C.c_void_p(oV.data_ptr()),
                                     C.c_void_p(idx.data_ptr()),
                                     C.c_void_p(counts.data_ptr()) if counts is not None else None,
                                     C.c_void_p(ws.data_ptr()), ws.numel(),
                                     C.c_void_p(torch.cuda.current_stream(K.device).cuda_stream)), "subgen_kcenter_compress")
    return oK, oV, idx, counts
