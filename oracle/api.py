"""numpy/ctypes front for the C oracle.  Test infrastructure only.

Every function takes one head at a time: ``Q, K, V`` are ``[N, D]`` float32
arrays (callers pass bf16-rounded values so the GPU sees the same numbers).
Results are float64.
"""
import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

SPATIAL, TEMPORAL, TEXTURAL, DENSE = 0, 1, 2, 3
SAMPLE_FIRST_FRAME, SAMPLE_EQUAL_INTERVAL = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rf_oracle.c")
_SO = os.path.join(_HERE, "librf_oracle.so")


class _CLayout(C.Structure):
    _fields_ = [("T", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("text_len", C.c_int32)]


class _CParams(C.Structure):
    _fields_ = [("bw_spatial", C.c_double), ("bw_temporal", C.c_double),
                ("tex_stride", C.c_int32), ("sample_interval", C.c_int32), ("two_head", C.c_int32),
                ("text_first", C.c_int32)]


@dataclass(frozen=True)
class Layout:
    """Latent video of T frames of H x W tokens, then text_len text tokens (Sec. 3.1)."""
    T: int
    H: int
    W: int
    text_len: int = 0

    def c(self):
        return _CLayout(self.T, self.H, self.W, self.text_len)


@dataclass(frozen=True)
class Params:
    """Pattern knobs: band widths (Sec. 4.1 default 1/4), checkerboard stride tau
    (default 2), global sampling interval omega (0 = T)."""
    bw_spatial: float = 0.25
    bw_temporal: float = 0.25
    tex_stride: int = 2
    sample_interval: int = 0
    two_head: bool = False
    text_first: bool = False  # the text tokens come before the video tokens instead of after

    def c(self):
        # the library takes the bandwidths as float32; promote those exact values
        return _CParams(float(np.float32(self.bw_spatial)), float(np.float32(self.bw_temporal)),
                        self.tex_stride, self.sample_interval, int(self.two_head), int(self.text_first))


def build(force=False):
    """Compile rf_oracle.c into librf_oracle.so (gcc, OpenMP). Returns the path."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-shared",
                               "-std=c11", "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        PL, PP = C.POINTER(_CLayout), C.POINTER(_CParams)
        f32p, f64p, i64p = C.POINTER(C.c_float), C.POINTER(C.c_double), C.POINTER(C.c_int64)
        lib.rfo_num_tokens.restype = C.c_int64
        lib.rfo_num_tokens.argtypes = [PL]
        lib.rfo_radius.restype = C.c_int64
        lib.rfo_radius.argtypes = [C.c_double, C.c_int64]
        lib.rfo_keep.restype = C.c_int
        lib.rfo_keep.argtypes = [C.c_int, C.c_int64, C.c_int64, PL, PP]
        lib.rfo_attention_rows.restype = None
        lib.rfo_attention_rows.argtypes = [f32p, f32p, f32p, C.c_int, C.c_int, PL, PP, i64p,
                                           C.c_int64, f64p, f64p]
        lib.rfo_attention_blockskip.restype = None
        lib.rfo_attention_blockskip.argtypes = [f32p, f32p, f32p, C.c_int, C.c_int, PL, PP, C.c_int,
                                                f64p, i64p, i64p]
        lib.rfo_sample_count.restype = C.c_int64
        lib.rfo_sample_count.argtypes = [PL, PP, C.c_int]
        lib.rfo_sample_token.restype = C.c_int64
        lib.rfo_sample_token.argtypes = [PL, PP, C.c_int, C.c_int64]
        lib.rfo_arm_recall.restype = C.c_double
        lib.rfo_arm_recall.argtypes = [f32p, f32p, C.c_int, PL, PP, C.c_int, C.c_int, f64p]
        lib.rfo_arm_classify.restype = C.c_int
        lib.rfo_arm_classify.argtypes = [f32p, f32p, C.c_int, PL, PP, C.c_int, C.c_double, f64p]
        lib.rfo_arm_classify_plus.restype = C.c_int
        lib.rfo_arm_classify_plus.argtypes = [f32p, f32p, C.c_int, PL, PP, C.c_int, C.c_double, f64p, C.c_int,
                                              C.POINTER(C.c_int), f64p]
        lib.rfo_decide.restype = C.c_int
        lib.rfo_decide.argtypes = [C.c_double, C.c_double, C.c_double]
        lib.rfo_keep_matrix.restype = None
        lib.rfo_keep_matrix.argtypes = [C.c_int, PL, PP, C.POINTER(C.c_uint8)]
        lib.rfo_kept_fraction.restype = C.c_double
        lib.rfo_kept_fraction.argtypes = [C.c_int, PL, PP]
        _lib = lib
    return _lib


def num_threads():
    """Threads the OpenMP loops will use (for reporting)."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    return len(os.sched_getaffinity(0))


def _f32(a, N, D):
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.shape == (N, D), (a.shape, N, D)
    return a


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def num_tokens(L):
    return int(_L().rfo_num_tokens(C.byref(L.c())))


def radius(bw, n):
    return int(_L().rfo_radius(float(np.float32(bw)), n))


def keep(cls, i, j, L, P=Params()):
    return bool(_L().rfo_keep(cls, i, j, C.byref(L.c()), C.byref(P.c())))


def keep_matrix(cls, L, P=Params()):
    """Boolean [N, N] mask by calling the token predicate pair by pair (small N only)."""
    N = num_tokens(L)
    M = np.zeros((N, N), dtype=np.uint8)
    _L().rfo_keep_matrix(cls, C.byref(L.c()), C.byref(P.c()), M.ctypes.data_as(C.POINTER(C.c_uint8)))
    return M.astype(bool)


def attention_rows(Q, K, V, cls, L, P, rows, want_prob=False):
    """Eq. 1-2 for the listed query rows. Returns O [len(rows), D] (and the softmax rows)."""
    N, D = num_tokens(L), Q.shape[-1]
    Q, K, V = _f32(Q, N, D), _f32(K, N, D), _f32(V, N, D)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows >= 0).all() and (rows < N).all()
    O = np.empty((len(rows), D), dtype=np.float64)
    Pr = np.empty((len(rows), N), dtype=np.float64) if want_prob else None
    _L().rfo_attention_rows(_p(Q, C.c_float), _p(K, C.c_float), _p(V, C.c_float), D, cls,
                            C.byref(L.c()), C.byref(P.c()), _p(rows, C.c_int64), len(rows),
                            _p(O, C.c_double), _p(Pr, C.c_double) if want_prob else None)
    return (O, Pr) if want_prob else O


def attention(Q, K, V, cls, L, P=Params()):
    """Eq. 1-2 for every query row of one head."""
    return attention_rows(Q, K, V, cls, L, P, np.arange(num_tokens(L)))


def attention_blockskip(Q, K, V, cls, L, P, block):
    """Block-skipping form. Returns (O [N, D], visited block pairs, total block pairs)."""
    N, D = num_tokens(L), Q.shape[-1]
    Q, K, V = _f32(Q, N, D), _f32(K, N, D), _f32(V, N, D)
    O = np.empty((N, D), dtype=np.float64)
    vis, tot = C.c_int64(0), C.c_int64(0)
    _L().rfo_attention_blockskip(_p(Q, C.c_float), _p(K, C.c_float), _p(V, C.c_float), D, cls,
                                 C.byref(L.c()), C.byref(P.c()), block, _p(O, C.c_double),
                                 C.byref(vis), C.byref(tot))
    return O, vis.value, tot.value


def sample_tokens(L, P, global_sampling):
    """Token indices of the ARM sample (Sec. 3.3): first frame, or every omega-th token."""
    lib, cl, cp = _L(), L.c(), P.c()
    n = lib.rfo_sample_count(C.byref(cl), C.byref(cp), int(global_sampling))
    return np.array([lib.rfo_sample_token(C.byref(cl), C.byref(cp), int(global_sampling), a)
                     for a in range(n)], dtype=np.int64)


def arm_recall(Q, K, L, P, global_sampling, cls, want_rows=False):
    """Eq. 6 on one head: mean over sampled rows of the softmax mass kept by the mask."""
    N, D = num_tokens(L), Q.shape[-1]
    Q, K = _f32(Q, N, D), _f32(K, N, D)
    cl, cp = L.c(), P.c()
    n = _L().rfo_sample_count(C.byref(cl), C.byref(cp), int(global_sampling))
    rr = np.empty(n, dtype=np.float64) if want_rows else None
    r = _L().rfo_arm_recall(_p(Q, C.c_float), _p(K, C.c_float), D, C.byref(cl), C.byref(cp),
                            int(global_sampling), cls, _p(rr, C.c_double) if want_rows else None)
    return (r, rr) if want_rows else r


def arm_classify(Q, K, L, P=Params(), sample_mode=SAMPLE_FIRST_FRAME, alpha=0.9):
    """Alg. 1 on one head. Returns (class, (R_hat, R_tilde))."""
    N, D = num_tokens(L), Q.shape[-1]
    Q, K = _f32(Q, N, D), _f32(K, N, D)
    rec = (C.c_double * 2)()
    c = _L().rfo_arm_classify(_p(Q, C.c_float), _p(K, C.c_float), D, C.byref(L.c()),
                              C.byref(P.c()), sample_mode, float(alpha), rec)
    return int(c), (rec[0], rec[1])


def arm_classify_plus(Q, K, L, P, sample_mode, alpha, bandwidths):
    """RainFusion+ on one head. Returns (class, bandwidth index or -1, recalls [2, n_bw])."""
    N, D = num_tokens(L), Q.shape[-1]
    Q, K = _f32(Q, N, D), _f32(K, N, D)
    bws = np.array([float(np.float32(b)) for b in bandwidths], dtype=np.float64)
    rec = np.empty((2, len(bws)), dtype=np.float64)
    idx = C.c_int(-2)
    c = _L().rfo_arm_classify_plus(_p(Q, C.c_float), _p(K, C.c_float), D, C.byref(L.c()), C.byref(P.c()),
                                   sample_mode, float(alpha), _p(bws, C.c_double), len(bws), C.byref(idx),
                                   _p(rec, C.c_double))
    return int(c), idx.value, rec


def decide(r_hat, r_tilde, alpha):
    return int(_L().rfo_decide(r_hat, r_tilde, alpha))


def kept_fraction(cls, L, P=Params()):
    return float(_L().rfo_kept_fraction(cls, C.byref(L.c()), C.byref(P.c())))
