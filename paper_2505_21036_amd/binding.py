"""ctypes binding of librainfusion.so: argument marshalling only.

Every function has the name and meaning of the C entry point it wraps (see
include/rainfusion.h).  Tensors are torch CUDA(HIP) tensors used purely as device
memory; kernels are enqueued on torch's current stream.  There is no fallback: if the
library has not been built, loading raises.
"""
import ctypes as C
import os

import numpy as np

RF_SPATIAL, RF_TEMPORAL, RF_TEXTURAL, RF_DENSE = 0, 1, 2, 3
RF_SAMPLE_FIRST_FRAME, RF_SAMPLE_EQUAL_INTERVAL = 0, 1
RF_FLAG_TWO_HEAD = 1
RF_FLAG_TEXT_FIRST = 2
RF_FLAG_FORCE_DENSE = 4
RF_FLAG_FIXED_ORDER = 8
RF_FLAG_WIDE_ROWS = 16
RF_PLAN_PARTIAL = 0x40000000
RF_KEY_TILE = 64
RF_LIST_TEMPORAL_POSITION_MAJOR = 4
RF_ATTENTION_MIN_WORKSPACE = 512
RF_ARM_STATIC_SCRATCH_BYTES = 2 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("RF_LIBRARY") or os.path.join(_HERE, "librainfusion.so")
_lib = None


class RfError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, rf_status_string(status), status))


class rf_layout(C.Structure):
    _fields_ = [("T", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("text_len", C.c_int32)]


class rf_params(C.Structure):
    _fields_ = [("bw_spatial", C.c_float), ("bw_temporal", C.c_float), ("tex_stride", C.c_int32),
                ("sample_interval", C.c_int32), ("flags", C.c_int32)]

    @classmethod
    def default(cls):
        return cls(0.25, 0.25, 2, 0, 0)


def library_path():
    return _LIB_PATH


def load_library():
    """Load librainfusion.so (built by paper_2505_21036_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("librainfusion.so is not built: run `python -m paper_2505_21036_amd.build` "
                           "(needs hipcc); there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    PL, PP, vp = C.POINTER(rf_layout), C.POINTER(rf_params), C.c_void_p
    lib.rf_version.restype = C.c_int
    lib.rf_version.argtypes = []
    lib.rf_status_string.restype = C.c_char_p
    lib.rf_status_string.argtypes = [C.c_int]
    lib.rf_arm_workspace_bytes.restype = C.c_size_t
    lib.rf_arm_workspace_bytes.argtypes = [C.c_int, C.c_int, PL, PP]
    lib.rf_arm_classify.restype = C.c_int
    lib.rf_arm_classify.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, PL, PP, C.c_int, C.c_float, vp, vp, vp,
                                    C.c_size_t, vp]
    lib.rf_arm_classify_noalloc.restype = C.c_int
    lib.rf_arm_classify_noalloc.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, PL, PP, C.c_int, C.c_float, vp, vp, vp]
    lib.rf_sparse_attention.restype = C.c_int
    lib.rf_sparse_attention.argtypes = [vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, PL, PP, C.c_int, vp, vp, C.c_size_t,
                                        vp]
    lib.rf_attention_workspace_bytes.restype = C.c_size_t
    lib.rf_attention_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, PL, PP]
    fp = C.POINTER(C.c_float)
    lib.rf_arm_classify_plus.restype = C.c_int
    lib.rf_arm_classify_plus.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, PL, PP, C.c_int, C.c_float, fp, C.c_int, vp,
                                         vp, vp, vp, C.c_size_t, vp]
    lib.rf_sparse_attention_plus.restype = C.c_int
    lib.rf_sparse_attention_plus.argtypes = [vp, vp, vp, vp, vp, fp, C.c_int, C.c_int, C.c_int, C.c_int, PL, PP, C.c_int,
                                             vp, vp, C.c_size_t, vp]
    lib.rf_plan_host.restype = C.c_int
    lib.rf_plan_host.argtypes = [PL, PP, C.c_int, C.c_int, vp, vp, C.c_size_t, C.POINTER(C.c_size_t)]
    lib.rf_plan_order.restype = C.c_int
    lib.rf_plan_order.argtypes = [PL, PP, C.c_int, C.c_int, vp, vp]
    lib.rf_plan_position_major.restype = C.c_int
    lib.rf_plan_position_major.argtypes = [PL, PP, vp]
    lib.rf_plan_clear.restype = C.c_int
    lib.rf_plan_clear.argtypes = []
    _lib = lib
    return lib


def rf_version():
    return load_library().rf_version()


def rf_status_string(status):
    return load_library().rf_status_string(status).decode()


def _pp(params):
    return None if params is None else C.byref(params)


def rf_arm_workspace_bytes(B, nH, layout, params=None):
    return load_library().rf_arm_workspace_bytes(B, nH, C.byref(layout), _pp(params))


def _check_bf16(t, name, shape=None):
    import torch
    if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 4):
        raise ValueError("%s must be a contiguous bf16 device tensor [B, nH, N, D]" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def rf_arm_classify(Q, K, layout, params=None, sample_mode=RF_SAMPLE_FIRST_FRAME, threshold=0.9,
                    head_class=None, recalls=None, workspace=None):
    """ARM (Alg. 1). Returns (head_class int32 [B, nH], recalls float32 [B, nH, 2]) on the device."""
    import torch
    _check_bf16(Q, "Q")
    _check_bf16(K, "K", Q.shape)
    B, nH, N, D = Q.shape
    if N != layout.T * layout.H * layout.W + layout.text_len:
        raise ValueError("N does not match the layout")
    if head_class is None:
        head_class = torch.empty(B, nH, dtype=torch.int32, device=Q.device)
    if recalls is None:
        recalls = torch.empty(B, nH, 2, dtype=torch.float32, device=Q.device)
    need = rf_arm_workspace_bytes(B, nH, layout, params)
    if workspace is None:
        workspace = torch.empty(max(need, 4), dtype=torch.uint8, device=Q.device)
    st = load_library().rf_arm_classify(Q.data_ptr(), K.data_ptr(), B, nH, D, C.byref(layout), _pp(params),
                                        sample_mode, threshold, head_class.data_ptr(), recalls.data_ptr(),
                                        workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                        _stream())
    if st != 0:
        raise RfError(st, "rf_arm_classify")
    return head_class, recalls


def rf_arm_classify_noalloc(Q, K, layout, params, sample_mode, threshold, head_class, recalls):
    """ARM (Alg. 1) without a workspace argument: per-row recalls go to the library's static scratch.
    head_class (int32 [B, nH]) and recalls (float32 [B, nH, 2]) are device tensors the caller provides,
    so the call allocates nothing."""
    _check_bf16(Q, "Q")
    _check_bf16(K, "K", Q.shape)
    B, nH, N, D = Q.shape
    if N != layout.T * layout.H * layout.W + layout.text_len:
        raise ValueError("N does not match the layout")
    st = load_library().rf_arm_classify_noalloc(Q.data_ptr(), K.data_ptr(), B, nH, D, C.byref(layout), _pp(params),
                                                sample_mode, threshold, head_class.data_ptr(), recalls.data_ptr(),
                                                _stream())
    if st != 0:
        raise RfError(st, "rf_arm_classify_noalloc")
    return head_class, recalls


def rf_arm_classify_plus(Q, K, layout, params, sample_mode, threshold, bandwidths):
    """RainFusion+ ARM. Returns (head_class [B, nH], head_bw [B, nH], recalls [B, nH, 2, n_bw]) on the device."""
    import torch
    _check_bf16(Q, "Q")
    _check_bf16(K, "K", Q.shape)
    B, nH, N, D = Q.shape
    if N != layout.T * layout.H * layout.W + layout.text_len:
        raise ValueError("N does not match the layout")
    n_bw = len(bandwidths)
    bws = (C.c_float * n_bw)(*bandwidths)
    head_class = torch.empty(B, nH, dtype=torch.int32, device=Q.device)
    head_bw = torch.empty(B, nH, dtype=torch.int32, device=Q.device)
    recalls = torch.empty(B, nH, 2, n_bw, dtype=torch.float32, device=Q.device)
    workspace = torch.empty(max(n_bw * rf_arm_workspace_bytes(B, nH, layout, params), 4), dtype=torch.uint8,
                            device=Q.device)
    st = load_library().rf_arm_classify_plus(Q.data_ptr(), K.data_ptr(), B, nH, D, C.byref(layout), _pp(params),
                                             sample_mode, threshold, bws, n_bw, head_class.data_ptr(),
                                             head_bw.data_ptr(), recalls.data_ptr(), workspace.data_ptr(),
                                             workspace.numel(), _stream())
    if st != 0:
        raise RfError(st, "rf_arm_classify_plus")
    return head_class, head_bw, recalls


def rf_sparse_attention_plus(Q, K, V, head_class, head_bw, bandwidths, layout, params=None, block=128, out=None,
                             workspace=None):
    """Sparse attention with per-head bandwidth (RainFusion+). head_bw: int32 device tensor [B, nH]."""
    import torch
    _check_bf16(Q, "Q")
    _check_bf16(K, "K", Q.shape)
    _check_bf16(V, "V", Q.shape)
    B, nH, N, D = Q.shape
    if N != layout.T * layout.H * layout.W + layout.text_len:
        raise ValueError("N does not match the layout")
    for t, name in ((head_class, "head_class"), (head_bw, "head_bw")):
        if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.numel() == B * nH):
            raise ValueError("%s must be a contiguous int32 device tensor with B*nH entries" % name)
    if out is None:
        out = torch.empty_like(Q)
    n_bw = len(bandwidths)
    bws = (C.c_float * n_bw)(*bandwidths)
    if workspace is None:  # the work-queue counters only: no packed copies
        workspace = torch.empty(RF_ATTENTION_MIN_WORKSPACE, dtype=torch.uint8, device=Q.device)
    ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    st = load_library().rf_sparse_attention_plus(Q.data_ptr(), K.data_ptr(), V.data_ptr(), head_class.data_ptr(),
                                                 head_bw.data_ptr(), bws, n_bw, B, nH, D, C.byref(layout), _pp(params),
                                                 block, out.data_ptr(), ws_ptr, ws_bytes, _stream())
    if st != 0:
        raise RfError(st, "rf_sparse_attention_plus")
    return out


def rf_attention_workspace_bytes(B, nH, D, layout, params=None):
    return load_library().rf_attention_workspace_bytes(B, nH, D, C.byref(layout), _pp(params))


def rf_sparse_attention(Q, K, V, head_class, layout, params=None, block=128, out=None, workspace=None):
    """Sparse attention forward (Eq. 1-5). head_class: int32 device tensor [B, nH] (may be None under
    RF_FLAG_FORCE_DENSE). Returns O.
    workspace: uint8 device tensor; with rf_attention_workspace_bytes() bytes the call packs K_C, V_C and
    position-major copies into it; None allocates the RF_ATTENTION_MIN_WORKSPACE bytes every call needs."""
    import torch
    _check_bf16(Q, "Q")
    _check_bf16(K, "K", Q.shape)
    _check_bf16(V, "V", Q.shape)
    B, nH, N, D = Q.shape
    if N != layout.T * layout.H * layout.W + layout.text_len:
        raise ValueError("N does not match the layout")
    if head_class is not None and not (head_class.is_cuda and head_class.dtype == torch.int32
                                       and head_class.is_contiguous() and head_class.numel() == B * nH):
        raise ValueError("head_class must be a contiguous int32 device tensor with B*nH entries")
    if out is None:
        out = torch.empty_like(Q)
    else:
        _check_bf16(out, "out", Q.shape)
    if workspace is None:  # the work-queue counters only: no packed copies
        workspace = torch.empty(RF_ATTENTION_MIN_WORKSPACE, dtype=torch.uint8, device=Q.device)
    ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    hc_ptr = None if head_class is None else head_class.data_ptr()
    st = load_library().rf_sparse_attention(Q.data_ptr(), K.data_ptr(), V.data_ptr(), hc_ptr, B, nH,
                                            D, C.byref(layout), _pp(params), block, out.data_ptr(), ws_ptr, ws_bytes,
                                            _stream())
    if st != 0:
        raise RfError(st, "rf_sparse_attention")
    return out


def rf_plan_host(layout, params, block, cls):
    """Host copy of one class's block list: (row_ptr int32 [nQB+1], cols int32 [nnz])."""
    lib = load_library()
    N = layout.T * layout.H * layout.W + layout.text_len
    nqb = (N + block - 1) // block
    row_ptr = np.zeros(nqb + 1, dtype=np.int32)
    needed = C.c_size_t(0)
    st = lib.rf_plan_host(C.byref(layout), _pp(params), block, cls, row_ptr.ctypes.data, None, 0, C.byref(needed))
    if st != 0:
        raise RfError(st, "rf_plan_host")
    cols = np.zeros(max(needed.value, 1), dtype=np.int32)
    st = lib.rf_plan_host(C.byref(layout), _pp(params), block, cls, row_ptr.ctypes.data, cols.ctypes.data,
                          cols.size, C.byref(needed))
    if st != 0:
        raise RfError(st, "rf_plan_host")
    return row_ptr, cols[:needed.value]


def rf_plan_order(layout, params, block, cls, full=False):
    """Order in which a head's query blocks are handed to workgroups: int32 permutation of 0..nQB-1.
    full=True: (order, first_entry int32 [nQB])."""
    N = layout.T * layout.H * layout.W + layout.text_len
    nqb = (N + block - 1) // block
    order = np.full(nqb, -1, dtype=np.int32)
    first = np.full(nqb, -1, dtype=np.int32)
    st = load_library().rf_plan_order(C.byref(layout), _pp(params), block, cls, order.ctypes.data, first.ctypes.data)
    if st != 0:
        raise RfError(st, "rf_plan_order")
    return (order, first) if full else order


def rf_plan_position_major(layout, params=None):
    """token_of[row] for the position-major order of the tokens (int32 [N])."""
    N = layout.T * layout.H * layout.W + layout.text_len
    out = np.full(N, -1, dtype=np.int32)
    st = load_library().rf_plan_position_major(C.byref(layout), _pp(params), out.ctypes.data)
    if st != 0:
        raise RfError(st, "rf_plan_position_major")
    return out


def plan_block_counts(layout, params, block, cls):
    """(visited (query block, key tile) pairs, of which partial, all such pairs) for one class:
    bookkeeping for FLOP counts; a pair stands for block x RF_KEY_TILE scores."""
    row_ptr, cols = rf_plan_host(layout, params, block, cls)
    N = layout.T * layout.H * layout.W + layout.text_len
    nqb, nkt = len(row_ptr) - 1, (N + RF_KEY_TILE - 1) // RF_KEY_TILE
    return int(len(cols)), int((cols & RF_PLAN_PARTIAL != 0).sum()), nqb * nkt


def rf_plan_clear():
    st = load_library().rf_plan_clear()
    if st != 0:
        raise RfError(st, "rf_plan_clear")
