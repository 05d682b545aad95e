"""ctypes binding of libqbert.so: argument marshalling only.

Every function has the name and meaning of the C entry point declared in include/qbert.h and
takes torch tensors that live on the GPU.  Outputs may be passed in (they are then written in
place) or are allocated here with torch; every step of the computation runs in the library's
HIP kernels on torch's current stream.  There is no fallback of any kind: if the shared
library has not been built, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqbert.so")
_lib = None

QB_K_ALIGN = 64
QB_N_BLOCK = 32
EXPORTS = ("qb_status_string", "qb_packed_nbytes", "qb_bwd_workspace_nbytes", "qb_workspace_nbytes", "qb_quantize_groupwise",
           "qb_quantize_groupwise_batched",
           "qb_quantize_act", "qb_quantize_act_batched", "qb_qlinear_fwd", "qb_qlinear_fwd_batched", "qb_qlinear_fwd_q8", "qb_qlinear_bwd_ste", "qb_qlinear_bwd_ste_static", "qb_unpack_codes",
           "qb_embedding_quantize", "qb_embedding_gather", "qb_embedding_quantize_bits", "qb_embedding_gather_bits",
           "qb_quantize_act_dyn", "qb_qlinear_fwd_dyn", "qb_quantize_groupwise_clip", "qb_quantize_act_dyn_tensor", "qb_qlinear_bwd_ste_masked",
           "qb_quantize_groupwise_asym", "qb_quantize_groupwise_asym_range", "qb_qlinear_fwd_asym", "qb_qlinear_fwd_asym_dyn", "qb_qlinear_bwd_ste_asym",
           "qb_power_iteration_scratch_floats", "qb_power_iteration", "qb_sensitivity_omega", "qb_rank_by_sensitivity",
           "qb_probe_mfma_i8")


# int hv(void *ctx, const float *v, float *out, void *stream)
HV_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p)


class _QuantJob(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("bits", ctypes.c_int),
                ("groups", ctypes.c_int), ("packed", ctypes.c_void_p), ("h", ctypes.c_void_p), ("m", ctypes.c_void_p),
                ("rs_w", ctypes.c_void_p)]


class _ActJob(ctypes.Structure):
    _fields_ = [("X", ctypes.c_void_p), ("T", ctypes.c_int64), ("K", ctypes.c_int64), ("clip", ctypes.c_float),
                ("Xq", ctypes.c_void_p), ("rs_x", ctypes.c_void_p)]


class _FwdJob(ctypes.Structure):
    _fields_ = [("Xq", ctypes.c_void_p), ("rs_x", ctypes.c_void_p), ("clip", ctypes.c_float), ("packed", ctypes.c_void_p),
                ("h", ctypes.c_void_p), ("rs_w", ctypes.c_void_p), ("bits", ctypes.c_int), ("groups", ctypes.c_int),
                ("T", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("bias", ctypes.c_void_p),
                ("Y", ctypes.c_void_p)]


class QBError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("qbert status %d: %s" % (status, message))
        self.status = status


def load_library():
    """Load libqbert.so; raises (never substitutes another implementation) if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libqbert.so is not built: run `python -m paper_1909_05840_amd.build` "
                           "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci, cf = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.qb_status_string.restype = ctypes.c_char_p
    lib.qb_status_string.argtypes = [ci]
    lib.qb_packed_nbytes.restype = ctypes.c_size_t
    lib.qb_packed_nbytes.argtypes = [i64, i64, ci]
    lib.qb_workspace_nbytes.restype = ctypes.c_size_t
    lib.qb_workspace_nbytes.argtypes = [ci, i64, i64, i64, ci]
    lib.qb_bwd_workspace_nbytes.restype = ctypes.c_size_t
    lib.qb_bwd_workspace_nbytes.argtypes = [i64, i64, i64]
    lib.qb_quantize_groupwise.restype = ci
    lib.qb_quantize_groupwise.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, vp]
    lib.qb_quantize_groupwise_batched.restype = ci
    lib.qb_quantize_groupwise_batched.argtypes = [ctypes.POINTER(_QuantJob), ci, vp]
    lib.qb_quantize_act.restype = ci
    lib.qb_quantize_act.argtypes = [vp, i64, i64, cf, vp, vp, vp]
    lib.qb_quantize_act_batched.restype = ci
    lib.qb_quantize_act_batched.argtypes = [ctypes.POINTER(_ActJob), ci, vp]
    lib.qb_qlinear_fwd.restype = ci
    lib.qb_qlinear_fwd.argtypes = [vp, vp, cf, vp, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.qb_qlinear_fwd_batched.restype = ci
    lib.qb_qlinear_fwd_batched.argtypes = [ctypes.POINTER(_FwdJob), ci, vp]
    lib.qb_qlinear_fwd_q8.restype = ci
    lib.qb_qlinear_fwd_q8.argtypes = [vp, vp, cf, vp, vp, vp, ci, ci, i64, i64, i64, vp, ci, cf, vp, vp, vp]
    lib.qb_qlinear_bwd_ste.restype = ci
    lib.qb_qlinear_bwd_ste.argtypes = [vp, vp, cf, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.qb_qlinear_bwd_ste_static.restype = ci
    lib.qb_qlinear_bwd_ste_static.argtypes = [vp, vp, cf, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp]
    lib.qb_quantize_groupwise_asym.restype = ci
    lib.qb_quantize_groupwise_asym.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, vp]
    lib.qb_quantize_groupwise_asym_range.restype = ci
    lib.qb_quantize_groupwise_asym_range.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.qb_qlinear_fwd_asym.restype = ci
    lib.qb_qlinear_fwd_asym.argtypes = [vp, vp, cf, vp, vp, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.qb_qlinear_fwd_asym_dyn.restype = ci
    lib.qb_qlinear_fwd_asym_dyn.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.qb_qlinear_bwd_ste_asym.restype = ci
    lib.qb_qlinear_bwd_ste_asym.argtypes = [vp, vp, cf, vp, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.qb_power_iteration_scratch_floats.restype = ctypes.c_size_t
    lib.qb_power_iteration_scratch_floats.argtypes = []
    lib.qb_power_iteration.restype = ci
    lib.qb_power_iteration.argtypes = [HV_FN, vp, i64, ci, vp, vp, vp, vp, vp]
    lib.qb_probe_mfma_i8.restype = ci
    lib.qb_probe_mfma_i8.argtypes = [ci, ci, vp, vp]
    lib.qb_sensitivity_omega.restype = ci
    lib.qb_sensitivity_omega.argtypes = [vp, ci, ci, vp]
    lib.qb_rank_by_sensitivity.restype = ci
    lib.qb_rank_by_sensitivity.argtypes = [vp, ci, vp]
    lib.qb_qlinear_bwd_ste_masked.restype = ci
    lib.qb_qlinear_bwd_ste_masked.argtypes = [vp, vp, cf, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.qb_unpack_codes.restype = ci
    lib.qb_unpack_codes.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.qb_embedding_quantize.restype = ci
    lib.qb_embedding_quantize.argtypes = [vp, i64, i64, ci, vp, vp, vp, vp]
    lib.qb_embedding_gather.restype = ci
    lib.qb_embedding_gather.argtypes = [vp, vp, i64, i64, ci, vp, i64, vp, vp]
    lib.qb_quantize_groupwise_clip.restype = ci
    lib.qb_quantize_groupwise_clip.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, vp]
    lib.qb_quantize_act_dyn.restype = ci
    lib.qb_quantize_act_dyn.argtypes = [vp, i64, i64, vp, vp, vp, vp]
    lib.qb_quantize_act_dyn_tensor.restype = ci
    lib.qb_quantize_act_dyn_tensor.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp]
    lib.qb_qlinear_fwd_dyn.restype = ci
    lib.qb_qlinear_fwd_dyn.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, i64, i64, i64, vp, vp, vp, vp]
    lib.qb_embedding_quantize_bits.restype = ci
    lib.qb_embedding_quantize_bits.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp]
    lib.qb_embedding_gather_bits.restype = ci
    lib.qb_embedding_gather_bits.argtypes = [vp, vp, i64, i64, ci, ci, vp, i64, vp, vp]
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise QBError(status, load_library().qb_status_string(status).decode())


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous %s tensor on the GPU" % (name, dtype))
    return t


def qb_status_string(status):
    return load_library().qb_status_string(int(status)).decode()


def qb_packed_nbytes(N, K, bits):
    return int(load_library().qb_packed_nbytes(N, K, bits))


QB_OP_QUANTIZE_GROUPWISE, QB_OP_QUANTIZE_ACT, QB_OP_QLINEAR_FWD, QB_OP_QLINEAR_BWD_STE, QB_OP_EMBEDDING, QB_OP_POWER_ITERATION = range(6)


def qb_workspace_nbytes(op, T, N, K, bits):
    return int(load_library().qb_workspace_nbytes(int(op), T, N, K, bits))


def qb_bwd_workspace_nbytes(T, N, K):
    return int(load_library().qb_bwd_workspace_nbytes(T, N, K))


def qb_quantize_groupwise(W, bits, groups, packed=None, h=None, m=None, rs_w=None):
    """W[N,K] fp32 -> (packed uint8 buffer, h[G], m[G], rs_w[N])."""
    lib = load_library()
    _dev(W, torch.float32, "W")
    N, K = W.shape
    dev = W.device
    if packed is None:
        packed = torch.empty(max(qb_packed_nbytes(N, K, bits), 1), dtype=torch.uint8, device=dev)
    if h is None:
        h = torch.empty(max(groups, 1), dtype=torch.float32, device=dev)
    if m is None:
        m = torch.empty(max(groups, 1), dtype=torch.float32, device=dev)
    if rs_w is None:
        rs_w = torch.empty(N, dtype=torch.int32, device=dev)
    _check(lib.qb_quantize_groupwise(_p(W), N, K, bits, groups, _p(packed), _p(h), _p(m), _p(rs_w), _stream()))
    return packed, h, m, rs_w


def qb_quantize_groupwise_batched(jobs):
    """jobs: list of dicts with W, bits, groups and optionally packed, h, m, rs_w (allocated here if absent).
    Returns the list of (packed, h, m, rs_w) tuples."""
    lib = load_library()
    arr = (_QuantJob * max(len(jobs), 1))()
    outs = []
    for i, j in enumerate(jobs):
        W = _dev(j["W"], torch.float32, "W")
        N, K = W.shape
        bits, groups = int(j["bits"]), int(j["groups"])
        dev = W.device
        packed = j.get("packed")
        if packed is None:
            packed = torch.empty(max(qb_packed_nbytes(N, K, bits), 1), dtype=torch.uint8, device=dev)
        h = j.get("h") if j.get("h") is not None else torch.empty(max(groups, 1), dtype=torch.float32, device=dev)
        m = j.get("m") if j.get("m") is not None else torch.empty(max(groups, 1), dtype=torch.float32, device=dev)
        rs = j.get("rs_w") if j.get("rs_w") is not None else torch.empty(N, dtype=torch.int32, device=dev)
        arr[i] = _QuantJob(W.data_ptr(), N, K, bits, groups, packed.data_ptr(), h.data_ptr(), m.data_ptr(), rs.data_ptr())
        outs.append((packed, h, m, rs))
    _check(lib.qb_quantize_groupwise_batched(arr, len(jobs), _stream()))
    return outs


def qb_quantize_act(X, clip, Xq=None, rs_x=None):
    """X[T,K] fp32 -> (Xq[T,K] int8, rs_x[T] int32)."""
    lib = load_library()
    _dev(X, torch.float32, "X")
    T, K = X.shape
    if Xq is None:
        Xq = torch.empty((T, K), dtype=torch.int8, device=X.device)
    if rs_x is None:
        rs_x = torch.empty(T, dtype=torch.int32, device=X.device)
    _check(lib.qb_quantize_act(_p(X), T, K, float(clip), _p(Xq), _p(rs_x), _stream()))
    return Xq, rs_x


def qb_quantize_act_batched(jobs):
    """jobs: list of dicts with X, clip and optionally Xq, rs_x (allocated here if absent): several tensors, one launch.
    Returns the list of (Xq, rs_x) tuples."""
    lib = load_library()
    arr = (_ActJob * max(len(jobs), 1))()
    outs = []
    for i, j in enumerate(jobs):
        X = _dev(j["X"], torch.float32, "X")
        T, K = X.shape
        Xq = j.get("Xq") if j.get("Xq") is not None else torch.empty((T, K), dtype=torch.int8, device=X.device)
        rs = j.get("rs_x") if j.get("rs_x") is not None else torch.empty(T, dtype=torch.int32, device=X.device)
        arr[i] = _ActJob(X.data_ptr(), T, K, float(j["clip"]), _dev(Xq, torch.int8, "Xq").data_ptr(),
                         _dev(rs, torch.int32, "rs_x").data_ptr())
        outs.append((Xq, rs))
    _check(lib.qb_quantize_act_batched(arr, len(jobs), _stream()))
    return outs


def qb_qlinear_fwd(Xq, rs_x, clip, packed, h, rs_w, bits, groups, N, bias=None, Y=None, A4_debug=None,
                   want_a4=False):
    """Integer product + de-quantization. Returns Y[T,N] fp32 (and A4[T,N] int32 if asked)."""
    lib = load_library()
    _dev(Xq, torch.int8, "Xq")
    T, K = Xq.shape
    if Y is None:
        Y = torch.empty((T, N), dtype=torch.float32, device=Xq.device)
    if want_a4 and A4_debug is None:
        A4_debug = torch.empty((T, N), dtype=torch.int32, device=Xq.device)
    _check(lib.qb_qlinear_fwd(_p(Xq), _p(rs_x), float(clip), _p(packed), _p(h), _p(rs_w), bits, groups,
                              T, N, K, _p(bias), _p(Y), _p(A4_debug), _stream()))
    return (Y, A4_debug) if A4_debug is not None else Y


def qb_qlinear_fwd_batched(jobs):
    """jobs: list of dicts with Xq, rs_x, clip, packed, h, rs_w, bits, groups, N and optionally bias, Y (allocated
    here if absent).  Independent linear layers, as few launches as possible.  Returns the list of Y tensors."""
    lib = load_library()
    arr = (_FwdJob * max(len(jobs), 1))()
    outs = []
    for i, j in enumerate(jobs):
        Xq = _dev(j["Xq"], torch.int8, "Xq")
        T, K = Xq.shape
        N = int(j["N"])
        Y = j.get("Y")
        if Y is None:
            Y = torch.empty((T, N), dtype=torch.float32, device=Xq.device)
        bias = j.get("bias")
        arr[i] = _FwdJob(Xq.data_ptr(), _dev(j["rs_x"], torch.int32, "rs_x").data_ptr(), float(j["clip"]),
                         _dev(j["packed"], torch.uint8, "packed").data_ptr(), _dev(j["h"], torch.float32, "h").data_ptr(),
                         _dev(j["rs_w"], torch.int32, "rs_w").data_ptr(), int(j["bits"]), int(j["groups"]), T, N, K,
                         _p(_dev(bias, torch.float32, "bias")) if bias is not None else None,
                         _dev(Y, torch.float32, "Y").data_ptr())
        outs.append(Y)
    _check(lib.qb_qlinear_fwd_batched(arr, len(jobs), _stream()))
    return outs


def qb_qlinear_fwd_q8(Xq, rs_x, clip, packed, h, rs_w, bits, groups, N, clip_out, bias=None, act=0, Yq=None,
                      rs_y=None):
    """Forward with the output quantized to 8 bits at once. Returns Yq[T,N] int8 (= u - 128), rs_y[T] int32."""
    lib = load_library()
    _dev(Xq, torch.int8, "Xq")
    T, K = Xq.shape
    if Yq is None:
        Yq = torch.empty((T, N), dtype=torch.int8, device=Xq.device)
    if rs_y is None:
        rs_y = torch.empty(T, dtype=torch.int32, device=Xq.device)
    _check(lib.qb_qlinear_fwd_q8(_p(Xq), _p(rs_x), float(clip), _p(packed), _p(h), _p(rs_w), bits, groups,
                                 T, N, K, _p(bias), int(act), float(clip_out), _p(Yq), _p(rs_y), _stream()))
    return Yq, rs_y


def qb_qlinear_bwd_ste(dY, Xq, clip, packed, h, bits, groups, want_dx=True, want_dw=True, dX=None, dW=None,
                       workspace=None):
    """dY[T,N] bf16 -> (dX[T,K] bf16 or None, dW[N,K] fp32 or None)."""
    lib = load_library()
    _dev(dY, torch.bfloat16, "dY")
    _dev(Xq, torch.int8, "Xq")
    T, N = dY.shape
    K = Xq.shape[1]
    dev = dY.device
    if want_dx and dX is None:
        dX = torch.empty((T, K), dtype=torch.bfloat16, device=dev)
    if want_dw and dW is None:
        dW = torch.empty((N, K), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(qb_bwd_workspace_nbytes(T, N, K), 256), dtype=torch.uint8, device=dev)
    _check(lib.qb_qlinear_bwd_ste(_p(dY), _p(Xq), float(clip), _p(packed), _p(h), bits, groups, T, N, K,
                                  _p(dX), _p(dW), _p(workspace), _stream()))
    return dX, dW


def qb_qlinear_bwd_ste_static(dY, Xq, clip, packed, h, bits, groups, dX=None, dW=None):
    """qb_qlinear_bwd_ste without a workspace (the library's fixed staging area); dX and dW are the caller's, or null
    to skip one of them.  The call itself allocates nothing."""
    lib = load_library()
    _dev(dY, torch.bfloat16, "dY")
    _dev(Xq, torch.int8, "Xq")
    T, N = dY.shape
    K = Xq.shape[1]
    _check(lib.qb_qlinear_bwd_ste_static(_p(dY), _p(Xq), float(clip), _p(packed), _p(h), bits, groups, T, N, K,
                                         _p(dX), _p(dW), _stream()))
    return dX, dW


def qb_qlinear_bwd_ste_masked(dY, Xq, clip, packed, h, bits, groups, X=None, W=None, m=None, want_dx=True,
                              want_dw=True, dX=None, dW=None, workspace=None):
    """The backward with the clamp's derivative: dX zero where |X| > clip (X given), dW zero where |W| > m of
    its group (W and m given)."""
    lib = load_library()
    _dev(dY, torch.bfloat16, "dY")
    _dev(Xq, torch.int8, "Xq")
    T, N = dY.shape
    K = Xq.shape[1]
    dev = dY.device
    if X is not None:
        _dev(X, torch.float32, "X")
        if tuple(X.shape) != (T, K):
            raise ValueError("X must be [T, K]")
    if W is not None:
        _dev(W, torch.float32, "W")
        if tuple(W.shape) != (N, K):
            raise ValueError("W must be [N, K]")
    if m is not None:
        _dev(m, torch.float32, "m")
        if m.numel() != groups:
            raise ValueError("m must hold one range per group")
    if want_dx and dX is None:
        dX = torch.empty((T, K), dtype=torch.bfloat16, device=dev)
    if want_dw and dW is None:
        dW = torch.empty((N, K), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(qb_bwd_workspace_nbytes(T, N, K), 256), dtype=torch.uint8, device=dev)
    _check(lib.qb_qlinear_bwd_ste_masked(_p(dY), _p(Xq), float(clip), _p(packed), _p(h), bits, groups, T, N, K,
                                         _p(X), _p(W), _p(m), _p(dX), _p(dW), _p(workspace), _stream()))
    return dX, dW


def qb_quantize_groupwise_asym(W, bits, groups, packed=None, delta=None, q0=None, rs_w=None):
    """Group ranges [min, max]: W[N,K] fp32 -> (packed, delta[G], q0[G], rs_w[N])."""
    lib = load_library()
    _dev(W, torch.float32, "W")
    N, K = W.shape
    dev = W.device
    if packed is None:
        packed = torch.empty(max(qb_packed_nbytes(N, K, bits), 1), dtype=torch.uint8, device=dev)
    if delta is None:
        delta = torch.empty(groups, dtype=torch.float32, device=dev)
    if q0 is None:
        q0 = torch.empty(groups, dtype=torch.float32, device=dev)
    if rs_w is None:
        rs_w = torch.empty(N, dtype=torch.int32, device=dev)
    _check(lib.qb_quantize_groupwise_asym(_p(W), N, K, bits, groups, _p(packed), _p(delta), _p(q0), _p(rs_w), _stream()))
    return packed, delta, q0, rs_w


def qb_quantize_groupwise_asym_range(W, bits, lo, hi, packed=None, delta=None, q0=None, rs_w=None):
    """Asymmetric group ranges [lo[g], hi[g]] given by the caller. Returns (packed, delta[G], q0[G], rs_w[N])."""
    lib = load_library()
    _dev(W, torch.float32, "W")
    _dev(lo, torch.float32, "lo")
    _dev(hi, torch.float32, "hi")
    N, K = W.shape
    groups = lo.numel()
    dev = W.device
    if packed is None:
        packed = torch.empty(max(qb_packed_nbytes(N, K, bits), 1), dtype=torch.uint8, device=dev)
    delta = delta if delta is not None else torch.empty(groups, dtype=torch.float32, device=dev)
    q0 = q0 if q0 is not None else torch.empty(groups, dtype=torch.float32, device=dev)
    rs_w = rs_w if rs_w is not None else torch.empty(N, dtype=torch.int32, device=dev)
    _check(lib.qb_quantize_groupwise_asym_range(_p(W), N, K, bits, groups, _p(lo), _p(hi), _p(packed), _p(delta), _p(q0),
                                                _p(rs_w), _stream()))
    return packed, delta, q0, rs_w


def qb_qlinear_fwd_asym(Xq, rs_x, clip, packed, delta, q0, rs_w, bits, groups, N, bias=None, Y=None, want_a4=False):
    """Forward with asymmetric group ranges. Returns Y[T,N] fp32 (and A4[T,N] int32 if asked)."""
    lib = load_library()
    _dev(Xq, torch.int8, "Xq")
    _dev(delta, torch.float32, "delta")
    _dev(q0, torch.float32, "q0")
    T, K = Xq.shape
    if Y is None:
        Y = torch.empty((T, N), dtype=torch.float32, device=Xq.device)
    A4 = torch.empty((T, N), dtype=torch.int32, device=Xq.device) if want_a4 else None
    _check(lib.qb_qlinear_fwd_asym(_p(Xq), _p(rs_x), float(clip), _p(packed), _p(delta), _p(q0), _p(rs_w), bits, groups,
                                   T, N, K, _p(bias), _p(Y), _p(A4), _stream()))
    return (Y, A4) if want_a4 else Y


def qb_qlinear_fwd_asym_dyn(Xq, rs_x, hx_rows, packed, delta, q0, rs_w, bits, groups, N, bias=None, Y=None, want_a4=False):
    """Forward with asymmetric group ranges and one activation scale per token. Returns Y (and A4 if asked)."""
    lib = load_library()
    _dev(Xq, torch.int8, "Xq")
    _dev(hx_rows, torch.float32, "hx_rows")
    _dev(delta, torch.float32, "delta")
    _dev(q0, torch.float32, "q0")
    T, K = Xq.shape
    if Y is None:
        Y = torch.empty((T, N), dtype=torch.float32, device=Xq.device)
    A4 = torch.empty((T, N), dtype=torch.int32, device=Xq.device) if want_a4 else None
    _check(lib.qb_qlinear_fwd_asym_dyn(_p(Xq), _p(rs_x), _p(hx_rows), _p(packed), _p(delta), _p(q0), _p(rs_w), bits, groups,
                                       T, N, K, _p(bias), _p(Y), _p(A4), _stream()))
    return (Y, A4) if want_a4 else Y


def qb_qlinear_bwd_ste_asym(dY, Xq, clip, packed, delta, q0, bits, groups, want_dx=True, want_dw=True, dX=None, dW=None,
                            workspace=None):
    """STE backward with asymmetric group ranges: dY[T,N] bf16 -> (dX[T,K] bf16 or None, dW[N,K] fp32 or None)."""
    lib = load_library()
    _dev(dY, torch.bfloat16, "dY")
    _dev(Xq, torch.int8, "Xq")
    T, N = dY.shape
    K = Xq.shape[1]
    dev = dY.device
    if want_dx and dX is None:
        dX = torch.empty((T, K), dtype=torch.bfloat16, device=dev)
    if want_dw and dW is None:
        dW = torch.empty((N, K), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(qb_bwd_workspace_nbytes(T, N, K), 256), dtype=torch.uint8, device=dev)
    _check(lib.qb_qlinear_bwd_ste_asym(_p(dY), _p(Xq), float(clip), _p(packed), _p(delta), _p(q0), bits, groups, T, N, K,
                                       _p(dX), _p(dW), _p(workspace), _stream()))
    return dX, dW


def qb_power_iteration(hv, v, iters, hv_buf=None, scratch=None, estimates=None):
    """Alg. 1.  hv(v, out) is a Python callable that enqueues out = H v on the current stream (v and out are the
    tensors given here); v[n] fp32 device is the start vector and is overwritten.  Returns (estimates[iters], v)."""
    lib = load_library()
    _dev(v, torch.float32, "v")
    n = v.numel()
    if hv_buf is None:
        hv_buf = torch.empty_like(v)
    if scratch is None:
        scratch = torch.empty(lib.qb_power_iteration_scratch_floats(), dtype=torch.float32, device=v.device)
    if estimates is None:
        estimates = torch.empty(iters, dtype=torch.float32, device=v.device)

    failure = []

    def trampoline(ctx, v_ptr, out_ptr, stream):
        if v_ptr != v.data_ptr() or out_ptr != hv_buf.data_ptr():
            return 1
        try:
            hv(v, hv_buf)
        except BaseException as exc:   # an exception must not cross the C frames: hand it over and stop the iteration
            failure.append(exc)
            return 1
        return 0
    cb = HV_FN(trampoline)
    rc = lib.qb_power_iteration(cb, None, n, iters, _p(v), _p(hv_buf), _p(scratch), _p(estimates), _stream())
    if failure:
        raise failure[0]
    _check(rc)
    return estimates, v


def qb_probe_mfma_i8(workgroups, iters, sink):
    """Enqueue the matrix-core issue-rate probe; returns the number of integer operations it performs."""
    lib = load_library()
    _check(lib.qb_probe_mfma_i8(int(workgroups), int(iters), _p(sink), _stream()))
    return workgroups * 4 * iters * 4 * 65536


def qb_sensitivity_omega(lambdas):
    """Eq. 2 on the host: lambdas[layers, runs] (numpy or nested lists) -> omega[layers] numpy fp32."""
    import numpy as np
    lib = load_library()
    lam = np.ascontiguousarray(lambdas, dtype=np.float32)
    layers, runs = lam.shape
    omega = np.empty(layers, np.float32)
    _check(lib.qb_sensitivity_omega(ctypes.c_void_p(lam.ctypes.data), layers, runs, ctypes.c_void_p(omega.ctypes.data)))
    return omega


def qb_rank_by_sensitivity(omega):
    """Layers by descending omega (host): numpy int32."""
    import numpy as np
    lib = load_library()
    om = np.ascontiguousarray(omega, dtype=np.float32)
    order = np.empty(om.shape[0], np.int32)
    _check(lib.qb_rank_by_sensitivity(ctypes.c_void_p(om.ctypes.data), om.shape[0], ctypes.c_void_p(order.ctypes.data)))
    return order


def qb_unpack_codes(packed, N, K, bits, codes=None):
    lib = load_library()
    if codes is None:
        codes = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(lib.qb_unpack_codes(_p(packed), N, K, bits, _p(codes), _stream()))
    return codes


def qb_embedding_quantize(E, groups, codes=None, h=None, m=None):
    lib = load_library()
    _dev(E, torch.float32, "E")
    V, d = E.shape
    if codes is None:
        codes = torch.empty((V, d), dtype=torch.uint8, device=E.device)
    if h is None:
        h = torch.empty(max(groups, 1), dtype=torch.float32, device=E.device)
    if m is None:
        m = torch.empty(max(groups, 1), dtype=torch.float32, device=E.device)
    _check(lib.qb_embedding_quantize(_p(E), V, d, groups, _p(codes), _p(h), _p(m), _stream()))
    return codes, h, m


def qb_embedding_gather(codes, h, groups, ids, out=None):
    lib = load_library()
    _dev(codes, torch.uint8, "codes")
    _dev(ids, torch.int64, "ids")
    V, d = codes.shape
    n = ids.shape[0]
    if out is None:
        out = torch.empty((n, d), dtype=torch.float32, device=codes.device)
    _check(lib.qb_embedding_gather(_p(codes), _p(h), V, d, groups, _p(ids), n, _p(out), _stream()))
    return out


def qb_embedding_quantize_bits(E, bits, groups, codes=None, h=None, m=None):
    """bits = 8: codes [V,d] uint8; bits = 4: codes [V,d/2], two codes per byte (even column in the low nibble)."""
    lib = load_library()
    _dev(E, torch.float32, "E")
    V, d = E.shape
    if codes is None:
        codes = torch.empty((V, d * bits // 8), dtype=torch.uint8, device=E.device)
    if h is None:
        h = torch.empty(max(groups, 1), dtype=torch.float32, device=E.device)
    if m is None:
        m = torch.empty(max(groups, 1), dtype=torch.float32, device=E.device)
    _check(lib.qb_embedding_quantize_bits(_p(E), V, d, bits, groups, _p(codes), _p(h), _p(m), _stream()))
    return codes, h, m


def qb_embedding_gather_bits(codes, h, bits, groups, ids, out=None):
    lib = load_library()
    _dev(codes, torch.uint8, "codes")
    _dev(ids, torch.int64, "ids")
    V = codes.shape[0]
    d = codes.shape[1] * 8 // bits
    n = ids.shape[0]
    if out is None:
        out = torch.empty((n, d), dtype=torch.float32, device=codes.device)
    _check(lib.qb_embedding_gather_bits(_p(codes), _p(h), V, d, bits, groups, _p(ids), n, _p(out), _stream()))
    return out


def qb_quantize_act_dyn(X, Xq=None, rs_x=None, hx_rows=None):
    """Per-token max-abs range: X[T,K] fp32 -> (Xq[T,K] int8, rs_x[T] int32, hx_rows[T] fp32)."""
    lib = load_library()
    _dev(X, torch.float32, "X")
    T, K = X.shape
    if Xq is None:
        Xq = torch.empty((T, K), dtype=torch.int8, device=X.device)
    if rs_x is None:
        rs_x = torch.empty(T, dtype=torch.int32, device=X.device)
    if hx_rows is None:
        hx_rows = torch.empty(T, dtype=torch.float32, device=X.device)
    _check(lib.qb_quantize_act_dyn(_p(X), T, K, _p(Xq), _p(rs_x), _p(hx_rows), _stream()))
    return Xq, rs_x, hx_rows


def qb_quantize_act_dyn_tensor(X, Xq=None, rs_x=None, hx_rows=None, c=None):
    """One max-abs range for the whole tensor: X[T,K] fp32 -> (Xq[T,K] int8, rs_x[T] int32, hx_rows[T] fp32 (all
    equal c/255), c[1] fp32 = max|X|)."""
    lib = load_library()
    _dev(X, torch.float32, "X")
    T, K = X.shape
    if Xq is None:
        Xq = torch.empty((T, K), dtype=torch.int8, device=X.device)
    if rs_x is None:
        rs_x = torch.empty(T, dtype=torch.int32, device=X.device)
    if hx_rows is None:
        hx_rows = torch.empty(T, dtype=torch.float32, device=X.device)
    if c is None:
        c = torch.empty(1, dtype=torch.float32, device=X.device)
    _check(lib.qb_quantize_act_dyn_tensor(_p(X), T, K, _p(Xq), _p(rs_x), _p(hx_rows), _p(c), _stream()))
    return Xq, rs_x, hx_rows, c


def qb_qlinear_fwd_dyn(Xq, rs_x, hx_rows, packed, h, rs_w, bits, groups, N, bias=None, Y=None, want_a4=False):
    """Forward with one activation scale per token. Returns Y[T,N] fp32 (and A4[T,N] int32 if asked)."""
    lib = load_library()
    _dev(Xq, torch.int8, "Xq")
    _dev(hx_rows, torch.float32, "hx_rows")
    T, K = Xq.shape
    if Y is None:
        Y = torch.empty((T, N), dtype=torch.float32, device=Xq.device)
    A4 = torch.empty((T, N), dtype=torch.int32, device=Xq.device) if want_a4 else None
    _check(lib.qb_qlinear_fwd_dyn(_p(Xq), _p(rs_x), _p(hx_rows), _p(packed), _p(h), _p(rs_w), bits, groups,
                                  T, N, K, _p(bias), _p(Y), _p(A4), _stream()))
    return (Y, A4) if want_a4 else Y


def qb_quantize_groupwise_clip(W, bits, m_in, packed=None, h=None, rs_w=None):
    """Group ranges [-m_in[g], +m_in[g]] given by the caller (device fp32 [G]). Returns (packed, h, rs_w)."""
    lib = load_library()
    _dev(W, torch.float32, "W")
    _dev(m_in, torch.float32, "m_in")
    N, K = W.shape
    G = m_in.shape[0]
    if packed is None:
        packed = torch.empty(max(qb_packed_nbytes(N, K, bits), 1), dtype=torch.uint8, device=W.device)
    if h is None:
        h = torch.empty(G, dtype=torch.float32, device=W.device)
    if rs_w is None:
        rs_w = torch.empty(N, dtype=torch.int32, device=W.device)
    _check(lib.qb_quantize_groupwise_clip(_p(W), N, K, bits, G, _p(m_in), _p(packed), _p(h), _p(rs_w), _stream()))
    return packed, h, rs_w
