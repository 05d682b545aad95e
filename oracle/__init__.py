"""CPU oracle for the group-wise quantized linear layer -- TEST INFRASTRUCTURE.

Thin numpy/ctypes front end of ``qbert_oracle.c``.  Only the tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the product package never does.
Every function takes and returns numpy arrays; nothing here knows about the GPU.
"""
import ctypes
import numpy as np

from . import build as _build

_I64 = ctypes.c_int64
_P = ctypes.c_void_p
_libs = {}


class OracleError(RuntimeError):
    pass


def _lib(openmp=False):
    if openmp not in _libs:
        _build.build()
        lib = ctypes.CDLL(_build.lib_path(openmp))
        lib.qbo_packed_row_bytes.restype = _I64
        lib.qbo_packed_row_bytes.argtypes = [_I64, ctypes.c_int]
        lib.qbo_num_threads.restype = ctypes.c_int
        _libs[openmp] = lib
    return _libs[openmp]


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc, what):
    if rc != 0:
        raise OracleError("%s failed with oracle status %d" % (what, rc))


def num_threads(openmp=True):
    return int(_lib(openmp).qbo_num_threads())


def quantize_groupwise(W, bits, groups):
    """Sec. 3.3 grouping + appendix quantizer. Returns codes[N,K] u8, h[G], m[G], rs_w[N]."""
    W = _c(W, np.float32)
    N, K = W.shape
    codes = np.empty((N, K), np.uint8)
    h = np.empty(groups, np.float32)
    m = np.empty(groups, np.float32)
    rs = np.empty(N, np.int32)
    rc = _lib().qbo_quantize_groupwise(_ptr(W), _I64(N), _I64(K), int(bits), _I64(groups),
                                       _ptr(codes), _ptr(h), _ptr(m), _ptr(rs))
    _check(rc, "quantize_groupwise")
    return codes, h, m, rs


def quantize_groupwise_clip(W, bits, m_in):
    """Group ranges [-m_in[g], +m_in[g]] given by the caller. Returns codes[N,K] u8, h[G] f32, rs_w[N] i32."""
    W = _c(W, np.float32)
    m_in = _c(m_in, np.float32)
    N, K = W.shape
    G = m_in.shape[0]
    codes = np.empty((N, K), np.uint8)
    h = np.empty(G, np.float32)
    rs = np.empty(N, np.int32)
    _check(_lib().qbo_quantize_groupwise_clip(_ptr(W), _I64(N), _I64(K), int(bits), _I64(G), _ptr(m_in), _ptr(codes),
                                              _ptr(h), _ptr(rs)), "quantize_groupwise_clip")
    return codes, h, rs


def dequantize_groupwise(codes, h, bits):
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    N, K = codes.shape
    out = np.empty((N, K), np.float64)
    _check(_lib().qbo_dequantize_groupwise(_ptr(codes), _ptr(h), _I64(N), _I64(K), int(bits),
                                           _I64(h.shape[0]), _ptr(out)), "dequantize_groupwise")
    return out


def packed_row_bytes(K, bits):
    return int(_lib().qbo_packed_row_bytes(_I64(K), int(bits)))


def pack(codes, bits):
    codes = _c(codes, np.uint8)
    N, K = codes.shape
    out = np.empty((N, packed_row_bytes(K, bits)), np.uint8)
    _check(_lib().qbo_pack(_ptr(codes), _I64(N), _I64(K), int(bits), _ptr(out)), "pack")
    return out


def unpack(packed, K, bits):
    packed = _c(packed, np.uint8)
    N = packed.shape[0]
    out = np.empty((N, K), np.uint8)
    _check(_lib().qbo_unpack(_ptr(packed), _I64(N), _I64(K), int(bits), _ptr(out)), "unpack")
    return out


def quantize_act(X, clip):
    """8-bit activation quantizer. Returns xq[T,K] int8 (= u-128) and rs_x[T] int32."""
    X = _c(X, np.float32)
    T, K = X.shape
    xq = np.empty((T, K), np.int8)
    rs = np.empty(T, np.int32)
    _check(_lib().qbo_quantize_act(_ptr(X), _I64(T), _I64(K), ctypes.c_float(clip), _ptr(xq), _ptr(rs)),
           "quantize_act")
    return xq, rs


def dequantize_act(xq, clip):
    xq = _c(xq, np.int8)
    T, K = xq.shape
    out = np.empty((T, K), np.float64)
    _check(_lib().qbo_dequantize_act(_ptr(xq), _I64(T), _I64(K), ctypes.c_float(clip), _ptr(out)),
           "dequantize_act")
    return out


def qlinear_fwd(xq, clip, codes, h, bits, bias=None, openmp=False):
    """Integer product + de-quantization. Returns Y[T,N] f32, A4[T,N] i32, acc[T,N] i32."""
    xq = _c(xq, np.int8)
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    T, K = xq.shape
    N = codes.shape[0]
    assert codes.shape[1] == K
    Y = np.empty((T, N), np.float32)
    A4 = np.empty((T, N), np.int32)
    acc = np.empty((T, N), np.int32)
    rc = _lib(openmp).qbo_qlinear_fwd(_ptr(xq), ctypes.c_float(clip), _ptr(codes), _ptr(h), int(bits),
                                      _I64(h.shape[0]), _I64(T), _I64(N), _I64(K), _ptr(bias),
                                      _ptr(Y), _ptr(A4), _ptr(acc))
    _check(rc, "qlinear_fwd")
    return Y, A4, acc


def quantize_act_dyn(X):
    """Per-token max-abs range. Returns xq[T,K] i8, rs_x[T] i32, hx[T] f32."""
    X = _c(X, np.float32)
    T, K = X.shape
    xq = np.empty((T, K), np.int8)
    rs = np.empty(T, np.int32)
    hx = np.empty(T, np.float32)
    _check(_lib().qbo_quantize_act_dyn(_ptr(X), _I64(T), _I64(K), _ptr(xq), _ptr(rs), _ptr(hx)), "quantize_act_dyn")
    return xq, rs, hx


def quantize_act_dyn_tensor(X):
    """One max-abs range for the whole tensor. Returns xq[T,K] i8, rs_x[T] i32, hx f32 (a scalar: c/255)."""
    X = _c(X, np.float32)
    T, K = X.shape
    xq = np.empty((T, K), np.int8)
    rs = np.empty(T, np.int32)
    hx = np.empty(1, np.float32)
    _check(_lib().qbo_quantize_act_dyn_tensor(_ptr(X), _I64(T), _I64(K), _ptr(xq), _ptr(rs), _ptr(hx)),
           "quantize_act_dyn_tensor")
    return xq, rs, hx[0]


def qlinear_fwd_dyn(xq, hx, codes, h, bits, bias=None, openmp=False):
    """Forward with one activation scale per token. Returns Y[T,N] f32, A4[T,N] i32."""
    xq = _c(xq, np.int8)
    hx = _c(hx, np.float32)
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    T, K = xq.shape
    N = codes.shape[0]
    Y = np.empty((T, N), np.float32)
    A4 = np.empty((T, N), np.int32)
    rc = _lib(openmp).qbo_qlinear_fwd_dyn(_ptr(xq), _ptr(hx), _ptr(codes), _ptr(h), int(bits), _I64(h.shape[0]),
                                          _I64(T), _I64(N), _I64(K), _ptr(bias), _ptr(Y), _ptr(A4))
    _check(rc, "qlinear_fwd_dyn")
    return Y, A4


def qlinear_fwd_q8(xq, clip, codes, h, bits, clip_out, bias=None, act=0, openmp=False):
    """Forward with the output quantized to 8 bits at once. Returns yq[T,N] i8 (= u - 128), rs_y[T] i32."""
    xq = _c(xq, np.int8)
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    T, K = xq.shape
    N = codes.shape[0]
    assert codes.shape[1] == K
    yq = np.empty((T, N), np.int8)
    rs_y = np.empty(T, np.int32)
    rc = _lib(openmp).qbo_qlinear_fwd_q8(_ptr(xq), ctypes.c_float(clip), _ptr(codes), _ptr(h), int(bits),
                                         _I64(h.shape[0]), _I64(T), _I64(N), _I64(K), _ptr(bias), int(act),
                                         ctypes.c_float(clip_out), _ptr(yq), _ptr(rs_y))
    _check(rc, "qlinear_fwd_q8")
    return yq, rs_y


def qlinear_fwd_sampled(xq, clip, codes, h, bits, ts, ns, bias=None):
    xq = _c(xq, np.int8)
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    ts = _c(ts, np.int64)
    ns = _c(ns, np.int64)
    T, K = xq.shape
    N = codes.shape[0]
    Y = np.empty(ts.shape[0], np.float32)
    A4 = np.empty(ts.shape[0], np.int32)
    rc = _lib().qbo_qlinear_fwd_sampled(_ptr(xq), ctypes.c_float(clip), _ptr(codes), _ptr(h), int(bits),
                                        _I64(h.shape[0]), _I64(T), _I64(N), _I64(K), _ptr(bias),
                                        _ptr(ts), _ptr(ns), _I64(ts.shape[0]), _ptr(Y), _ptr(A4))
    _check(rc, "qlinear_fwd_sampled")
    return Y, A4


def qlinear_bwd_ste(dY_bf16, xq, clip, codes, h, bits, want_dx=True, want_dw=True, openmp=False):
    """STE backward in binary64. dY_bf16 holds bfloat16 bit patterns (uint16)."""
    dY = _c(dY_bf16, np.uint16)
    xq = _c(xq, np.int8)
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    T, K = xq.shape
    N = codes.shape[0]
    assert dY.shape == (T, N)
    dX = np.empty((T, K), np.float64) if want_dx else None
    dW = np.empty((N, K), np.float64) if want_dw else None
    rc = _lib(openmp).qbo_qlinear_bwd_ste(_ptr(dY), _ptr(xq), ctypes.c_float(clip), _ptr(codes), _ptr(h),
                                          int(bits), _I64(h.shape[0]), _I64(T), _I64(N), _I64(K),
                                          _ptr(dX), _ptr(dW))
    _check(rc, "qlinear_bwd_ste")
    return dX, dW


def qlinear_bwd_ste_masked(dY_bf16, xq, clip, codes, h, bits, X=None, W=None, m=None, want_dx=True, want_dw=True,
                           openmp=False):
    """STE backward with the clamp's derivative: dX zero where |X| > clip, dW zero where |W| > m of its group."""
    dY = _c(dY_bf16, np.uint16)
    xq = _c(xq, np.int8)
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    X = None if X is None else _c(X, np.float32)
    W = None if W is None else _c(W, np.float32)
    m = None if m is None else _c(m, np.float32)
    T, K = xq.shape
    N = codes.shape[0]
    assert dY.shape == (T, N) and (X is None or X.shape == (T, K)) and (W is None or W.shape == (N, K))
    assert m is None or m.shape == h.shape
    dX = np.empty((T, K), np.float64) if want_dx else None
    dW = np.empty((N, K), np.float64) if want_dw else None
    rc = _lib(openmp).qbo_qlinear_bwd_ste_masked(_ptr(dY), _ptr(xq), ctypes.c_float(clip), _ptr(codes), _ptr(h),
                                                 int(bits), _I64(h.shape[0]), _I64(T), _I64(N), _I64(K),
                                                 _ptr(X), _ptr(W), _ptr(m), _ptr(dX), _ptr(dW))
    _check(rc, "qlinear_bwd_ste_masked")
    return dX, dW


def bwd_dx_sampled(dY_bf16, codes, h, bits, ts, js):
    dY = _c(dY_bf16, np.uint16)
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    ts = _c(ts, np.int64)
    js = _c(js, np.int64)
    T, N = dY.shape
    K = codes.shape[1]
    out = np.empty(ts.shape[0], np.float64)
    rc = _lib().qbo_bwd_dx_sampled(_ptr(dY), _ptr(codes), _ptr(h), int(bits), _I64(h.shape[0]),
                                   _I64(T), _I64(N), _I64(K), _ptr(ts), _ptr(js), _I64(ts.shape[0]), _ptr(out))
    _check(rc, "bwd_dx_sampled")
    return out


def bwd_dw_sampled(dY_bf16, xq, clip, ns, js):
    dY = _c(dY_bf16, np.uint16)
    xq = _c(xq, np.int8)
    ns = _c(ns, np.int64)
    js = _c(js, np.int64)
    T, N = dY.shape
    K = xq.shape[1]
    out = np.empty(ns.shape[0], np.float64)
    rc = _lib().qbo_bwd_dw_sampled(_ptr(dY), _ptr(xq), ctypes.c_float(clip), _I64(T), _I64(N), _I64(K),
                                   _ptr(ns), _ptr(js), _I64(ns.shape[0]), _ptr(out))
    _check(rc, "bwd_dw_sampled")
    return out


def embedding_quantize(E, groups, bits=8):
    """Codes u8 [V,d] (0..2^bits-1), h[G], m[G]; bits is 8 or 4."""
    E = _c(E, np.float32)
    V, d = E.shape
    codes = np.empty((V, d), np.uint8)
    h = np.empty(groups, np.float32)
    m = np.empty(groups, np.float32)
    _check(_lib().qbo_embedding_quantize_bits(_ptr(E), _I64(V), _I64(d), int(bits), _I64(groups), _ptr(codes),
                                              _ptr(h), _ptr(m)), "embedding_quantize")
    return codes, h, m


def embedding_gather(codes, h, ids, bits=8):
    codes = _c(codes, np.uint8)
    h = _c(h, np.float32)
    ids = _c(ids, np.int64)
    V, d = codes.shape
    out = np.empty((ids.shape[0], d), np.float64)
    _check(_lib().qbo_embedding_gather_bits(_ptr(codes), _ptr(h), _I64(V), _I64(d), int(bits), _I64(h.shape[0]),
                                            _ptr(ids), _I64(ids.shape[0]), _ptr(out)), "embedding_gather")
    return out


def quantize_groupwise_asym(W, bits, groups):
    """Group ranges [min, max] of the data. Returns codes[N,K] u8, delta[G] f32, q0[G] f32, rs_w[N] i32."""
    W = _c(W, np.float32)
    N, K = W.shape
    codes = np.empty((N, K), np.uint8)
    delta = np.empty(groups, np.float32)
    q0 = np.empty(groups, np.float32)
    rs = np.empty(N, np.int32)
    _check(_lib().qbo_quantize_groupwise_asym(_ptr(W), _I64(N), _I64(K), int(bits), _I64(groups), _ptr(codes),
                                              _ptr(delta), _ptr(q0), _ptr(rs)), "quantize_groupwise_asym")
    return codes, delta, q0, rs


def quantize_groupwise_asym_range(W, bits, lo, hi):
    """Caller-given group ranges [lo[g], hi[g]] (App.: a sub-interval of the data's range; weights outside are clamped).
    Returns (codes[N,K] u8, delta[G] f32, q0[G] f32, rs_w[N] i32)."""
    W = _c(W, np.float32)
    lo = _c(lo, np.float32)
    hi = _c(hi, np.float32)
    N, K = W.shape
    G = lo.shape[0]
    codes = np.empty((N, K), np.uint8)
    delta = np.empty(G, np.float32)
    q0 = np.empty(G, np.float32)
    rs_w = np.empty(N, np.int32)
    _check(_lib().qbo_quantize_groupwise_asym_range(_ptr(W), _I64(N), _I64(K), int(bits), _I64(G), _ptr(lo), _ptr(hi),
                                                    _ptr(codes), _ptr(delta), _ptr(q0), _ptr(rs_w)),
           "quantize_groupwise_asym_range")
    return codes, delta, q0, rs_w


def dequantize_groupwise_asym(codes, delta, q0):
    codes = _c(codes, np.uint8)
    delta = _c(delta, np.float32)
    q0 = _c(q0, np.float32)
    N, K = codes.shape
    Wq = np.empty((N, K), np.float64)
    _check(_lib().qbo_dequantize_groupwise_asym(_ptr(codes), _ptr(delta), _ptr(q0), _I64(N), _I64(K),
                                                _I64(delta.shape[0]), _ptr(Wq)), "dequantize_groupwise_asym")
    return Wq


def qlinear_fwd_asym(xq, clip, codes, delta, q0, bias=None, want_s=False, openmp=False):
    """Forward with asymmetric weights. Returns Y[T,N] f32 (and S[T,N] i64 if asked)."""
    xq = _c(xq, np.int8)
    codes = _c(codes, np.uint8)
    delta = _c(delta, np.float32)
    q0 = _c(q0, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    T, K = xq.shape
    N = codes.shape[0]
    assert codes.shape[1] == K
    Y = np.empty((T, N), np.float32)
    S = np.empty((T, N), np.int64) if want_s else None
    _check(_lib(openmp).qbo_qlinear_fwd_asym(_ptr(xq), ctypes.c_float(clip), _ptr(codes), _ptr(delta), _ptr(q0),
                                             _I64(delta.shape[0]), _I64(T), _I64(N), _I64(K), _ptr(bias), _ptr(Y),
                                             _ptr(S)), "qlinear_fwd_asym")
    return (Y, S) if want_s else Y


def qlinear_fwd_asym_dyn(xq, hx, codes, delta, q0, bias=None, openmp=False):
    """Forward with asymmetric weights and one activation scale per token. Returns Y[T,N] f32."""
    xq = _c(xq, np.int8)
    hx = _c(hx, np.float32)
    codes = _c(codes, np.uint8)
    delta = _c(delta, np.float32)
    q0 = _c(q0, np.float32)
    bias = None if bias is None else _c(bias, np.float32)
    T, K = xq.shape
    N = codes.shape[0]
    assert codes.shape[1] == K and hx.shape == (T,)
    Y = np.empty((T, N), np.float32)
    _check(_lib(openmp).qbo_qlinear_fwd_asym_dyn(_ptr(xq), _ptr(hx), _ptr(codes), _ptr(delta), _ptr(q0),
                                                 _I64(delta.shape[0]), _I64(T), _I64(N), _I64(K), _ptr(bias), _ptr(Y)),
           "qlinear_fwd_asym_dyn")
    return Y


def qlinear_bwd_dx_asym(dY_bf16, codes, delta, q0, openmp=False):
    dY = _c(dY_bf16, np.uint16)
    codes = _c(codes, np.uint8)
    delta = _c(delta, np.float32)
    q0 = _c(q0, np.float32)
    T, N = dY.shape
    K = codes.shape[1]
    dX = np.empty((T, K), np.float64)
    _check(_lib(openmp).qbo_qlinear_bwd_dx_asym(_ptr(dY), _ptr(codes), _ptr(delta), _ptr(q0), _I64(delta.shape[0]),
                                                _I64(T), _I64(N), _I64(K), _ptr(dX)), "qlinear_bwd_dx_asym")
    return dX



# ---- Hessian-based sensitivity (Sec. 3.2, Eq. 2; Alg. 1) -- plain numpy, binary64 ---------------------------------
def sensitivity_omega(lams):
    """Eq. 2: Omega_i = |mean(lambda_i)| + std(lambda_i) over the runs of layer i (population standard deviation).
    lams[layers, runs] -> omega[layers]."""
    lams = np.asarray(lams, np.float64)
    return np.abs(lams.mean(axis=1)) + lams.std(axis=1)


def rank_by_sensitivity(omega):
    """Layers in descending order of Omega (Sec. 3.2: sorted in descending order); equal values keep layer order."""
    omega = np.asarray(omega, np.float64)
    return np.argsort(-omega, kind="stable").astype(np.int32)


def power_iteration(hv, v0, iters):
    """Alg. 1 with the Hessian-vector product as a callable: v = v0/|v0|; n times: Hv = hv(v), the step's eigenvalue
    estimate v.Hv (v has unit length), v = Hv/|Hv|.  Returns (estimates[iters], v)."""
    v = np.asarray(v0, np.float64)
    v = v / np.sqrt((v * v).sum())
    lam = np.empty(iters, np.float64)
    for i in range(iters):
        Hv = np.asarray(hv(v), np.float64)
        lam[i] = (v * Hv).sum()
        nrm = np.sqrt((Hv * Hv).sum())
        if nrm == 0.0:
            lam[i:] = 0.0
            break
        v = Hv / nrm
    return lam, v
