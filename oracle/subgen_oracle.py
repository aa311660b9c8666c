"""ctypes front-end of the SubGen CPU oracle (``subgen_oracle.c``).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests, the smoke check and the
bench's cpu-baseline leg may import this module.  It shares nothing with the
HIP library and never imports the product package.

The arithmetic lives in the C file (Algorithm 1 of the paper in representative
mode plus the sliding window of Section 3.2); this file only builds it with
gcc, marshals numpy arrays in and copies state out.  ``exact_attention`` is
the textbook definition (Eq. 1) written with numpy in float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "subgen_oracle.c"
_LIB = _HERE / "libsubgen_oracle.so"
_lib = None


GCC_FLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c99", "-shared", "-fPIC"]


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (no fast-math, no FMA contraction)."""
    override = os.environ.get("SUBGEN_ORACLE_LIB")      # the mutation test points the wrapper at a doctored build
    if override:
        return Path(override)
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", *GCC_FLAGS, "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    L = C.CDLL(str(build()))
    P = C.c_void_p
    fp = C.POINTER(C.c_float)
    dp = C.POINTER(C.c_double)
    L.sgo_create.restype = P
    L.sgo_create.argtypes = [C.c_int, C.c_double, C.c_int, C.c_int, C.c_uint64, C.c_uint32, C.c_int, C.c_int]
    L.sgo_destroy.argtypes = [P]
    L.sgo_update.argtypes = [P, fp, fp]
    L.sgo_attend.restype = C.c_int
    L.sgo_attend.argtypes = [P, fp, dp, dp, dp]
    L.sgo_ingest.argtypes = [P, fp, fp, C.c_int64]
    L.sgo_decode.restype = C.c_int
    L.sgo_decode.argtypes = [P, fp, fp, fp, C.c_int64, C.c_int, dp]
    L.sgo_uniform24.restype = C.c_float
    L.sgo_uniform24.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32]
    L.sgo_uniform24_res.restype = C.c_float
    L.sgo_uniform24_res.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32]
    L.sgo_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
    L.sgo_set_overrides.restype = C.c_int
    L.sgo_set_overrides.argtypes = [P, C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.c_int64]
    L.sgo_overrides_used.restype = C.c_int64
    L.sgo_overrides_used.argtypes = [P]
    for name, rt in [("sgo_m", C.c_int), ("sgo_n_seen", C.c_int64), ("sgo_n_evicted", C.c_int64),
                     ("sgo_mu", C.c_double), ("sgo_overflowed", C.c_int), ("sgo_dropped", C.c_int64)]:
        getattr(L, name).restype = rt
        getattr(L, name).argtypes = [P]
    for name in ["sgo_centers", "sgo_reservoirs", "sgo_counts", "sgo_sample_k", "sgo_sample_v", "sgo_sample_idx", "sgo_sample_vn",
                 "sgo_window_k", "sgo_window_v", "sgo_window_idx", "sgo_assign", "sgo_created", "sgo_dist1",
                 "sgo_dist2"]:
        getattr(L, name).restype = P
        getattr(L, name).argtypes = [P]
    _lib = L
    return L


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _fptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def philox4x32_10(ctr, key):
    L = _load()
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    L.sgo_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def uniform24(seed: int, stream: int, token: int, slot: int) -> float:
    return float(_load().sgo_uniform24(seed, stream, token, slot))


def uniform24_res(seed: int, stream: int, token: int, slot: int) -> float:
    """Coin of reservoir slot `slot` of the cluster that `token` joins (t >= 1)."""
    return float(_load().sgo_uniform24_res(seed, stream, token, slot))


class OracleStream:
    """One (sequence, layer, head) stream of the oracle."""

    def __init__(self, d: int, delta: float, s: int, w: int, seed: int = 0, stream: int = 0,
                 max_centers: int = 0, t: int = 0):
        self._L = _load()
        # delta is a float32 at the library boundary; the oracle squares its double value
        self.delta = float(np.float32(delta))
        self.d, self.s, self.w, self.t = int(d), int(s), int(w), int(t)
        self._h = self._L.sgo_create(self.d, self.delta, self.s, self.w, int(seed), int(stream), int(max_centers),
                                     self.t)
        if not self._h:
            raise ValueError("invalid oracle parameters")

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            self._L.sgo_destroy(h)

    FORCE_NEW = -2

    def set_overrides(self, overrides: dict) -> None:
        """Near-tie protocol: force the clustering decision of some tokens ({token: cluster index to join, or
        FORCE_NEW}).  Only a parity harness that has checked the decision margin calls this, before any update."""
        toks = np.array(sorted(overrides), dtype=np.int64)
        decs = np.array([overrides[int(t)] for t in toks], dtype=np.int32)
        rc = self._L.sgo_set_overrides(self._h, toks.ctypes.data_as(C.POINTER(C.c_int64)),
                                       decs.ctypes.data_as(C.POINTER(C.c_int32)), len(toks))
        if rc:
            raise ValueError("bad override list (or the stream has already seen tokens)")

    @property
    def overrides_used(self) -> int:
        return int(self._L.sgo_overrides_used(self._h))

    # -- the three operations ------------------------------------------------
    def update(self, k, v) -> None:
        k, v = _f32(k), _f32(v)
        assert k.shape == (self.d,) and v.shape == (self.d,)
        self._L.sgo_update(self._h, _fptr(k), _fptr(v))

    def ingest(self, K, V) -> None:
        K, V = _f32(K), _f32(V)
        assert K.ndim == 2 and K.shape[1] == self.d and V.shape == K.shape
        self._L.sgo_ingest(self._h, _fptr(K), _fptr(V), K.shape[0])

    def attend(self, q, return_den: bool = False):
        q = _f32(q)
        assert q.shape == (self.d,)
        out = np.empty(self.d, dtype=np.float64)
        den = C.c_double()
        mx = C.c_double()
        rc = self._L.sgo_attend(self._h, _fptr(q), out.ctypes.data_as(C.POINTER(C.c_double)), C.byref(den),
                                C.byref(mx))
        if rc:
            raise RuntimeError("attend before any token")
        if return_den:
            return out, den.value, mx.value
        return out

    def decode(self, K, V, Q) -> np.ndarray:
        """update(K[t],V[t]) then attend(Q[t,h]) for every t; Q is [n,g,d] or [n,d]."""
        K, V, Q = _f32(K), _f32(V), _f32(Q)
        if Q.ndim == 2:
            Q = Q[:, None, :]
        n, g = Q.shape[0], Q.shape[1]
        out = np.empty((n, g, self.d), dtype=np.float64)
        rc = self._L.sgo_decode(self._h, _fptr(K), _fptr(V), _fptr(np.ascontiguousarray(Q)), n, g,
                                out.ctypes.data_as(C.POINTER(C.c_double)))
        if rc:
            raise RuntimeError("attend before any token")
        return out

    # -- state read-out (copies) --------------------------------------------
    def _arr(self, fn, dtype, shape):
        n = int(np.prod(shape))
        if n == 0:
            return np.zeros(shape, dtype=dtype)
        p = getattr(self._L, fn)(self._h)
        buf = (C.c_char * (n * np.dtype(dtype).itemsize)).from_address(p)
        return np.frombuffer(buf, dtype=dtype).reshape(shape).copy()

    @property
    def m(self) -> int:
        return self._L.sgo_m(self._h)

    @property
    def n_seen(self) -> int:
        return self._L.sgo_n_seen(self._h)

    @property
    def n_evicted(self) -> int:
        return self._L.sgo_n_evicted(self._h)

    @property
    def mu(self) -> float:
        return self._L.sgo_mu(self._h)

    @property
    def overflowed(self) -> bool:
        return bool(self._L.sgo_overflowed(self._h))

    @property
    def dropped(self) -> int:
        """Tokens with NaN/Inf (or a squared norm beyond fp32) dropped when they left the window."""
        return int(self._L.sgo_dropped(self._h))

    @property
    def centers(self):
        return self._arr("sgo_centers", np.float32, (self.m, self.d))

    @property
    def reservoirs(self):
        """Per-cluster reservoirs S_i as [m, t, d] (t >= 1)."""
        return self._arr("sgo_reservoirs", np.float32, (self.m, self.t, self.d))

    @property
    def counts(self):
        return self._arr("sgo_counts", np.int64, (self.m,))

    @property
    def sample_k(self):
        return self._arr("sgo_sample_k", np.float32, (self.s, self.d))

    @property
    def sample_v(self):
        return self._arr("sgo_sample_v", np.float32, (self.s, self.d))

    @property
    def sample_idx(self):
        return self._arr("sgo_sample_idx", np.int64, (self.s,))

    @property
    def sample_vn(self):
        return self._arr("sgo_sample_vn", np.float32, (self.s,))

    @property
    def window_fill(self) -> int:
        return min(self.n_seen, self.w)

    @property
    def window_k(self):
        """Window rows in ring-slot order (slot = token index mod w)."""
        return self._arr("sgo_window_k", np.float32, (self.w, self.d))[: self.window_fill]

    @property
    def window_v(self):
        return self._arr("sgo_window_v", np.float32, (self.w, self.d))[: self.window_fill]

    @property
    def window_idx(self):
        return self._arr("sgo_window_idx", np.int64, (self.w,))[: self.window_fill]

    @property
    def assign(self):
        return self._arr("sgo_assign", np.int32, (self.n_evicted,))

    @property
    def created(self):
        return self._arr("sgo_created", np.uint8, (self.n_evicted,))

    @property
    def dist1(self):
        """Squared distance of each evicted token to its nearest representative (inf for the first)."""
        return self._arr("sgo_dist1", np.float64, (self.n_evicted,))

    @property
    def dist2(self):
        return self._arr("sgo_dist2", np.float64, (self.n_evicted,))

    def margins(self):
        """Relative decision margins per evicted token.

        thr: abs(dist - delta)/delta of the nearest representative (inf when there was
        none, or delta == 0 and dist > 0); gap: (d2 - d1)/d1 on distances when the
        runner-up is also within delta (else inf).
        """
        d1 = np.sqrt(self.dist1)
        d2 = np.sqrt(self.dist2)
        with np.errstate(divide="ignore", invalid="ignore"):
            thr = np.where(np.isfinite(d1), np.abs(d1 - self.delta) / self.delta, np.inf)
            thr = np.where(np.isnan(thr), 0.0, thr)
            gap = np.where(np.isfinite(d2) & (d2 <= self.delta), (d2 - d1) / d1, np.inf)
            gap = np.where(np.isnan(gap), 0.0, gap)
        return thr, gap


def exact_attention(K, V, q) -> np.ndarray:
    """softmax(K q)^T V in float64 (Eq. 1 of the paper), max-shifted."""
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    sc = K @ q
    e = np.exp(sc - sc.max())
    return (e @ V) / e.sum()


def greedy_kcenter(K, k: int):
    """Farthest-point traversal (the greedy k-center algorithm the paper applies once, Section 3.2) in float64.

    First center = point 0; every next center = the point farthest from the centers chosen so far (lowest index
    on ties).  Returns (indices of the centers in selection order, nearest-center assignment of every point with
    the lowest center on ties, squared distance of every point to its nearest center).
    """
    K = np.asarray(K, dtype=np.float64)
    n = K.shape[0]
    kk = min(int(k), n)
    sel, assign, mind = [], np.zeros(n, dtype=np.int64), np.full(n, np.inf)
    c = 0
    for it in range(kk):
        sel.append(c)
        dist = ((K - K[c]) ** 2).sum(axis=1)
        closer = dist < mind
        assign[closer] = it
        mind = np.where(closer, dist, mind)
        c = int(np.argmax(mind))          # first occurrence of the maximum
    return np.array(sel, dtype=np.int64), assign, mind


def kcenter_compress(K, V, k: int, r: int):
    """k centers among the tokens older than the r most recent, then those r tokens (Section 3.2)."""
    K, V = np.asarray(K), np.asarray(V)
    n = K.shape[0]
    rwin = min(r, n)
    nold = n - rwin
    sel, assign, _ = greedy_kcenter(K[:nold], k) if nold > 0 else (np.zeros(0, np.int64), np.zeros(0, np.int64), None)
    idx = np.full(k + r, -1, dtype=np.int64)
    idx[: len(sel)] = sel
    idx[k: k + rwin] = np.arange(nold, n)
    counts = np.bincount(assign, minlength=k)[:k] if nold > 0 else np.zeros(k, dtype=np.int64)
    return idx, counts
